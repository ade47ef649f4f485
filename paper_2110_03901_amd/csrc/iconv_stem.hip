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
// contiguous range of TH x TW output blocks.  The four waves read the next block's input patch
// into registers before the current block's MFMAs and park it in the other of two LDS patch
// buffers after the current block's stores; the only synchronisation is one barrier per block.
// The layer is bound by the write of y, which goes through a wave-private LDS staging area so that
// every store instruction covers whole cache lines.  Two workgroups of four waves share a compute
// unit (two waves per SIMD), which leaves each wave 256 vector registers.  A second form (stem_sw_kernel
// below) gives the stores to waves of their own and is the one chosen once a compute unit has three or more
// blocks to work through.
#include <atomic>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

struct StemGeom {
    int TH, TW_LOG2;     // output block: TH rows, TW = 1 << TW_LOG2 (16 or 32) columns
    int PH, PPAIRS;      // patch rows, 16-byte pixel pairs per patch row (the row pitch)
    int PPAIRS_USED;     // pairs of a patch row that hold pixels; the rest is padding that is never read
    int tiles_h, tiles_w, tiles_n;
    int total_tiles;
    int tiles_base, tiles_rem;   // workgroup i owns tiles_base (+1 if i < tiles_rem) consecutive blocks
    int shift;           // 1 when pad is odd: the 8-pixel run starts one pixel left of tap 0
    int b_bytes;         // LDS bytes of the weights (R * 4 KiB)
    int patch_bytes;     // LDS bytes of one patch buffer (whole workgroup-wide pieces)
    float inv_ppairs;    // 1 / PPAIRS
};

constexpr int kStemBN = 64;
constexpr int kStemWaves = 4;
constexpr int kStemPatchItems = 4;   // 16-byte patch pieces per lane at most (patch <= 16 KiB)

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
__global__ void __launch_bounds__(kStemWaves * 64)
stem_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const StemGeom g) {
    typedef typename Elem<T>::frag frag_t;
    // [weights: (r, k-chunk 0..3, filter 0..63) x 16 B][patch 0][patch 1][output staging: 4 KiB per compute
    // wave], a patch = (row, pixel pair) x 16 B
    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int TW = 1 << g.TW_LOG2;

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    // ranges differ by at most one tile
    const int t_begin = wg * g.tiles_base + min(wg, g.tiles_rem);
    const int t_end = t_begin + g.tiles_base + (wg < g.tiles_rem ? 1 : 0);
    // All tiles of a workgroup's range must use the same filters for the resident weights to be
    // valid: the host only makes ranges that do (tiles_n == 1), or ranges of one tile.
    const int k0 = stem_decode(t_begin, g).k0;

    // ---- patch loads: lane-constant part.  Piece i of the lane is pixel pair (i * 256 + tid) of the
    // patch in row-major (row, pair) order.  A pair never straddles the image edge (W and the patch
    // origin column are even), so a pair is either loaded whole or zero.
    const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * 8u;
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
    const int npairs = g.PH * g.PPAIRS;
    int p_h[kStemPatchItems], p_w[kStemPatchItems];       // patch row and column (in pixels) of the piece; column << 0: none
#pragma unroll
    for (int i = 0; i < kStemPatchItems; ++i) {
        const int pi = i * (kStemWaves * 64) + tid;
        const int ph = (int)(((float)pi + 0.5f) * g.inv_ppairs);
        const bool used = pi < npairs && pi - ph * g.PPAIRS < g.PPAIRS_USED;
        p_h[i] = used ? ph : 0;
        p_w[i] = used ? 2 * (pi - ph * g.PPAIRS) : -(1 << 30);
    }
    auto load_patch = [&](int tile, u32x4 (&regs)[kStemPatchItems]) {
        const StemTile tc = stem_decode(tile, g);
        const int h_org = tc.p0 * s.stride - s.pad;                 // input row of patch row 0
        const int w_org = tc.q0 * s.stride - s.pad - g.shift;       // input column of patch column 0 (even)
        const int base = (tc.n * s.H + h_org) * s.W + w_org;        // may be negative; in-range sums are not
#pragma unroll
        for (int i = 0; i < kStemPatchItems; ++i) {
            if (i * (kStemWaves * 64) < npairs) {                   // uniform
                const int h = h_org + p_h[i], ww = w_org + p_w[i];
                const bool ok = ((unsigned)h < (unsigned)s.H) & ((unsigned)ww < (unsigned)s.W);
                const uint32_t off = (uint32_t)(base + p_h[i] * s.W + p_w[i]) * 8u;
                regs[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, ok ? off : x_bytes, 0, 0));
            }
        }
    };
    auto park_patch = [&](int buf, const u32x4 (&regs)[kStemPatchItems]) {
        u32x4* dst = lds + ((g.b_bytes + buf * g.patch_bytes) >> 4) + tid;
#pragma unroll
        for (int i = 0; i < kStemPatchItems; ++i)
            if (i * (kStemWaves * 64) < npairs) dst[i * (kStemWaves * 64)] = regs[i];
    };
    u32x4 pregs[kStemPatchItems];
    load_patch(t_begin, pregs);                 // in flight while the weights are laid out

    // ---- weights, once: w[k][r][s][0..3] (8 bytes) -> slot (s + shift) of filter row r: 16-byte
    // chunk (s + shift)/2, half (s + shift)%2; the other slots are zero.  Chunk-major, so that the
    // 32 lanes of an operand read touch consecutive 16-byte words; filter k of (r, chunk) sits at
    // k ^ ((4r + chunk) & 15), which keeps those reads a permutation of consecutive words and
    // spreads the tap writes below (consecutive lanes = consecutive taps of one filter, which
    // would otherwise all fall into the same banks) over the banks.  Index arithmetic divides by
    // multiplying with a reciprocal in fp32: (i + 0.5) / d is never closer than 0.5 / d to an
    // integer, far more than the rounding error at these sizes (i < 2^13, d <= 80).
    {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        uint2* b8 = reinterpret_cast<uint2*>(lds);
        constexpr int nthreads = kStemWaves * 64;
        // the padding slots of the 8-pixel runs (filter fastest)
        const int npad = 8 - s.S;
        const float inv_npad = npad > 0 ? 1.0f / (float)npad : 0.f;
        for (int it = tid; it < kStemBN * s.R * npad; it += nthreads) {
            const int k = it & (kStemBN - 1);
            const int rj = it >> 6;
            const int r = (int)(((float)rj + 0.5f) * inv_npad), jj = rj - r * npad;
            const int j = jj < g.shift ? jj : jj + s.S;
            const int rc = r * 4 + (j >> 1);
            b8[((rc * kStemBN + (k ^ (rc & 15))) << 1) + (j & 1)] = uint2{0u, 0u};
        }
        // the taps, read in memory order (coalesced), sixteen loads in flight per thread; filters
        // beyond K read as zero (offset past the end of the buffer)
        const int RS = s.R * s.S;
        const int items = kStemBN * RS;
        const float inv_rs = 1.0f / (float)RS, inv_s = 1.0f / (float)s.S;
        const uint32_t w_bytes = (uint32_t)s.K * RS * 8u;
        const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
        const uint32_t w_base = (uint32_t)k0 * RS * 8u;
        for (int base = tid; base < items; base += nthreads * 16) {
            u32x2 v[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int it = base + u * nthreads;
                v[u] = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(
                                                     w_rsrc, it < items ? w_base + (uint32_t)it * 8u : w_bytes, 0, 0));
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int it = base + u * nthreads;
                const int k = (int)(((float)it + 0.5f) * inv_rs);
                const int rs = it - k * RS;
                const int r = (int)(((float)rs + 0.5f) * inv_s), j = rs - r * s.S + g.shift;
                const int rc = r * 4 + (j >> 1);
                if (it < items) b8[((rc * kStemBN + (k ^ (rc & 15))) << 1) + (j & 1)] = uint2{v[u].x, v[u].y};
            }
        }
    }

    // ---- per-lane constants of the block loop
    // Everything that depends only on the lane is computed once, so that a block costs few
    // vector instructions besides its LDS reads, MFMAs and stores.
    const int frow = lane & 31, fk = lane >> 5;
    const int npx = g.TH * TW;
    constexpr int BM = kStemWaves * MI * 32;
    const char* lds_b = reinterpret_cast<const char*>(lds);
    uint32_t a_off[MI];                           // byte offset in the patch of the lane's run at filter row 0
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int t = (wave * MI + mi) * 32 + frow;
        const int th = t >> g.TW_LOG2, tw = t & (TW - 1);
        a_off[mi] = (uint32_t)(t < npx ? th * s.stride * g.PPAIRS + tw * (s.stride >> 1) + fk : fk) * 16u;
    }
    // weights of (r, kk, ni): chunk 2kk + fk, filter 32ni + frow at slot (frow ^ ((4r + 2kk + fk) & 15)) =
    // ((frow ^ fk) ^ ((4r + 2kk) & 15)): a lane constant xor a uniform
    const uint32_t b_off = (uint32_t)(fk * kStemBN) * 16u;
    const uint32_t b_lane = (uint32_t)(frow ^ fk) * 16u;
    const uint32_t row_bytes = (uint32_t)g.PPAIRS * 16u;
    // which of the lane's two pixels per K slice are padding positions of the run; their weights
    // are zero, but the input there is zeroed too so that a non-finite neighbour cannot leak in
    bool zero_lo[2], zero_hi[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int j = 4 * kk + 2 * fk;
        zero_lo[kk] = j < g.shift || j >= s.S + g.shift;
        zero_hi[kk] = (j + 1) < g.shift || (j + 1) >= s.S + g.shift;
    }
    const bool mask_kk0 = g.shift != 0 || s.S + g.shift < 4;      // uniform: slice kk holds a padding slot
    const bool mask_kk1 = s.S + g.shift < 8;
    const bool vec_ok = (s.K & 3) == 0;

    // Output staging (vec_ok): each 32-pixel x 32-filter fragment goes through a 4 KiB area private
    // to the wave, so that 8 lanes store one pixel's 128 contiguous bytes (a whole cache line)
    // instead of 32 lanes storing 32 bytes of 32 different lines.  The 16-byte piece c of pixel t
    // sits at stage_off(t, c): neither the deposit (8 lanes of a write pass = 8 pixels, one piece) nor the
    // read-back (16 lanes of a read pass = 2 pixels, 8 pieces) has a bank conflict.  LDS operations of
    // one wave execute in order, so no wait is needed between deposit and read-back.
    char* stg = reinterpret_cast<char*>(lds) + g.b_bytes + 2 * g.patch_bytes + wave * 4096;
    const int c8 = lane & 7, l3 = lane >> 3;
    uint32_t sw[4];                               // deposit offset per filter quad
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) sw[gq] = stage_off(frow, 2 * gq + fk);
    const uint32_t sr = stage_off(l3, c8);        // read-back: piece l%8 of pixel l/8 (+ 8j: 1024 bytes further on)
    // the lane's piece of pixel 8j + l/8 of fragment mi lies at y_lane + (a uniform offset of (mi, j))
    // bytes from the block's origin: 8j + l/8 < 32 <= 32 * (fragment index), and TW is 16 or 32
    const uint32_t y_lane = (uint32_t)(l3 * s.K + 4 * c8) * (uint32_t)sizeof(TO);
    bool k_ok[2];
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) k_ok[ni] = k0 + ni * 32 + 4 * c8 + 3 < s.K;
    const size_t y_elems = (size_t)s.M * s.K;

    park_patch(0, pregs);
    __syncthreads();                            // weights and patch 0 are in LDS
    for (int tile = t_begin; tile < t_end; ++tile) {
        if (tile + 1 < t_end) load_patch(tile + 1, pregs);
        const char* pa = lds_b + g.b_bytes + ((tile - t_begin) & 1) * g.patch_bytes;
        const char* pb = lds_b + b_off;
        floatx16 acc[MI][2];
        frag_t a0[MI], b0[2], a1[MI], b1[2];    // operands of the two K slices of a filter row

        auto fetch = [&](int r, int kk, frag_t (&af)[MI], frag_t (&bf)[2]) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
                af[mi] = *reinterpret_cast<const frag_t*>(pa + a_off[mi] + (uint32_t)r * row_bytes + kk * 32);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                bf[ni] = *reinterpret_cast<const frag_t*>(pb + (b_lane ^ (uint32_t)(((4 * r + 2 * kk) & 15) << 4)) + r * 4096 +
                                                          kk * 2048 + ni * 512);
        };
        auto mma = [&](frag_t (&af)[MI], frag_t (&bf)[2], int kk, bool first) {
            if (kk == 0 ? mask_kk0 : mask_kk1) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) {
                    u32x4 v = __builtin_bit_cast(u32x4, af[mi]);
                    if (zero_lo[kk]) { v.x = 0u; v.y = 0u; }
                    if (zero_hi[kk]) { v.z = 0u; v.w = 0u; }
                    af[mi] = __builtin_bit_cast(frag_t, v);
                }
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    if (first) {
                        floatx16 z;
#pragma unroll
                        for (int v = 0; v < 16; ++v) z[v] = 0.f;
                        acc[mi][ni] = Elem<T>::mfma32(bf[ni], af[mi], z);
                    } else {
                        acc[mi][ni] = Elem<T>::mfma32(bf[ni], af[mi], acc[mi][ni]);
                    }
                }
        };
        // the operands of the next use of a slice are read from LDS while the other slice's MFMAs run
        // (the fetch after the last row re-reads that row: unconditional, so that the number of LDS
        // reads in flight is known at every wait)
        const int r_last = s.R - 1;
        fetch(0, 0, a0, b0);
        fetch(0, 1, a1, b1);
        mma(a0, b0, 0, true);
        fetch(min(1, r_last), 0, a0, b0);
        mma(a1, b1, 1, false);
        for (int r = 1; r < s.R; ++r) {
            fetch(r, 1, a1, b1);
            mma(a0, b0, 0, false);
            fetch(min(r + 1, r_last), 0, a0, b0);
            mma(a1, b1, 1, false);
        }

        // ---- epilogue: lane l holds block pixel 32*frag + l%32 and, in accumulator element v, filter
        // 8*(v/4) + 4*(l/32) + v%4 of the 32-wide block (the filters are the MFMA's row operand).
        const StemTile tc = stem_decode(tile, g);
        if (vec_ok) {
            // stores go through a buffer descriptor that starts at the block's first output
            const size_t org = ((size_t)(tc.n * s.P + tc.p0) * s.Q + tc.q0) * s.K + k0;
            const size_t rem = (y_elems - org) * sizeof(TO);
            const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + org, 0, rem > 0xffffffffull ? 0xffffffffu : (uint32_t)rem,
                                                                   kRsrcFlags);
            const bool edge = npx < BM || tc.p0 + g.TH > s.P || tc.q0 + TW > s.Q;    // uniform
            // deposits and read-backs of all fragments are issued back to back through the same 4 KiB
            // (in order within the wave), the stores follow as the read-backs arrive
            u32x4 out[MI][2][4];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        u32x4 v;
                        v.x = __float_as_uint(acc[mi][ni][4 * gq]);     v.y = __float_as_uint(acc[mi][ni][4 * gq + 1]);
                        v.z = __float_as_uint(acc[mi][ni][4 * gq + 2]); v.w = __float_as_uint(acc[mi][ni][4 * gq + 3]);
                        *reinterpret_cast<u32x4*>(stg + sw[gq]) = v;
                    }
                    __builtin_amdgcn_wave_barrier();
#pragma unroll
                    for (int j = 0; j < 4; ++j) out[mi][ni][j] = *reinterpret_cast<const u32x4*>(stg + sr + j * 1024);
                }
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
                for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        bool ok = k_ok[ni];
                        if (edge) {
                            const int t = (wave * MI + mi) * 32 + 8 * j + l3;
                            ok = ok && t < npx && tc.p0 + (t >> g.TW_LOG2) < s.P && tc.q0 + (t & (TW - 1)) < s.Q;
                        }
                        const int t0 = (wave * MI + mi) * 32 + 8 * j;       // uniform
                        const uint32_t y_uni = (uint32_t)(((t0 >> g.TW_LOG2) * s.Q + (t0 & (TW - 1))) * s.K + ni * 32) * (uint32_t)sizeof(TO);
                        if (ok) store_piece<TO>(out[mi][ni][j], y_rsrc, y_lane + y_uni);
                    }
                }
            }
        } else {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int t = (wave * MI + mi) * 32 + frow;
                const int p = tc.p0 + (t >> g.TW_LOG2), q = tc.q0 + (t & (TW - 1));
                if (t < npx && p < s.P && q < s.Q) {
                    TO* yrow = y + (size_t)((tc.n * s.P + p) * s.Q + q) * s.K;
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int col = k0 + ni * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                            if (col < s.K) yrow[col] = to_out<TO>(acc[mi][ni][v]);
                        }
                }
            }
        }
        // the other buffer was last read for the previous block, which every wave finished before
        // the barrier that ended it
        if (tile + 1 < t_end) park_patch((tile + 1 - t_begin) & 1, pregs);
        __syncthreads();                        // next patch is in LDS; this block's buffer may be refilled
    }
}

// ---- the same kernel with STORE WAVES: eight compute waves (one 32-pixel fragment each, 256 pixels per block)
// and four store waves in one workgroup per compute unit.  A wave that stores is held until the memory system
// has taken its data, and this layer is bound by the write of y: here the compute waves deposit their fragments
// in a 64 KiB staging area (fragment f, filter half ni at (2f + ni) * 4 KiB, layout stage_off) and go on with
// the next block, while the store waves, which took the area into registers at the start of the tick, write the
// previous block out.  Two barriers per block: S (the block's deposits are complete, the next patch is parked)
// and M (the store waves hold the previous block in registers, the area may be overwritten).
constexpr int kSwCompute = 8, kSwStore = 4, kSwWaves = kSwCompute + kSwStore;
constexpr int kSwPatchItems = 2;                 // 16-byte patch pieces per compute lane at most (patch <= 16 KiB)
constexpr int kSwStageBytes = kSwCompute * 2 * 4096;

template <typename T, typename TO>
__global__ void __launch_bounds__(kSwWaves * 64)
stem_sw_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const StemGeom g) {
    typedef typename Elem<T>::frag frag_t;
    // [weights][patch 0][patch 1][output staging: 8 fragments x 2 filter halves x 4 KiB]
    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int TW = 1 << g.TW_LOG2;
    constexpr int CT = kSwCompute * 64;         // compute threads: they load and park the patches

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int t_begin = wg * g.tiles_base + min(wg, g.tiles_rem);
    const int t_end = t_begin + g.tiles_base + (wg < g.tiles_rem ? 1 : 0);
    const int k0 = stem_decode(t_begin, g).k0;
    const bool computes = wave < kSwCompute;

    // ---- patch loads (compute waves): piece i of the lane is pixel pair (i * 512 + tid)
    const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * 8u;
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
    const int npairs = g.PH * g.PPAIRS;
    int p_h[kSwPatchItems], p_w[kSwPatchItems];
#pragma unroll
    for (int i = 0; i < kSwPatchItems; ++i) {
        const int pi = i * CT + tid;
        const int ph = (int)(((float)pi + 0.5f) * g.inv_ppairs);
        const bool used = computes && pi < npairs && pi - ph * g.PPAIRS < g.PPAIRS_USED;
        p_h[i] = used ? ph : 0;
        p_w[i] = used ? 2 * (pi - ph * g.PPAIRS) : -(1 << 30);
    }
    auto load_patch = [&](int tile, u32x4 (&regs)[kSwPatchItems]) {
        const StemTile tc = stem_decode(tile, g);
        const int h_org = tc.p0 * s.stride - s.pad;
        const int w_org = tc.q0 * s.stride - s.pad - g.shift;
        const int base = (tc.n * s.H + h_org) * s.W + w_org;
#pragma unroll
        for (int i = 0; i < kSwPatchItems; ++i) {
            if (i * CT < npairs) {                                  // uniform
                const int h = h_org + p_h[i], ww = w_org + p_w[i];
                const bool ok = ((unsigned)h < (unsigned)s.H) & ((unsigned)ww < (unsigned)s.W);
                const uint32_t off = (uint32_t)(base + p_h[i] * s.W + p_w[i]) * 8u;
                regs[i] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, ok ? off : x_bytes, 0, 0));
            }
        }
    };
    auto park_patch = [&](int buf, const u32x4 (&regs)[kSwPatchItems]) {
        u32x4* dst = lds + ((g.b_bytes + buf * g.patch_bytes) >> 4) + tid;
#pragma unroll
        for (int i = 0; i < kSwPatchItems; ++i)
            if (i * CT < npairs && i * CT + tid < (g.patch_bytes >> 4)) dst[i * CT] = regs[i];
    };
    u32x4 pregs[kSwPatchItems];
    if (computes) load_patch(t_begin, pregs);

    // ---- weights, once, by all waves (the layout of the kernel above)
    {
        typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
        uint2* b8 = reinterpret_cast<uint2*>(lds);
        constexpr int nthreads = kSwWaves * 64;
        const int npad = 8 - s.S;
        const float inv_npad = npad > 0 ? 1.0f / (float)npad : 0.f;
        for (int it = tid; it < kStemBN * s.R * npad; it += nthreads) {
            const int k = it & (kStemBN - 1);
            const int rj = it >> 6;
            const int r = (int)(((float)rj + 0.5f) * inv_npad), jj = rj - r * npad;
            const int j = jj < g.shift ? jj : jj + s.S;
            const int rc = r * 4 + (j >> 1);
            b8[((rc * kStemBN + (k ^ (rc & 15))) << 1) + (j & 1)] = uint2{0u, 0u};
        }
        const int RS = s.R * s.S;
        const int items = kStemBN * RS;
        const float inv_rs = 1.0f / (float)RS, inv_s = 1.0f / (float)s.S;
        const uint32_t w_bytes = (uint32_t)s.K * RS * 8u;
        const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
        const uint32_t w_base = (uint32_t)k0 * RS * 8u;
        for (int base = tid; base < items; base += nthreads * 8) {
            u32x2 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int it = base + u * nthreads;
                v[u] = __builtin_bit_cast(u32x2, __builtin_amdgcn_raw_buffer_load_b64(
                                                    w_rsrc, it < items ? w_base + (uint32_t)it * 8u : w_bytes, 0, 0));
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int it = base + u * nthreads;
                const int k = (int)(((float)it + 0.5f) * inv_rs);
                const int rs = it - k * RS;
                const int r = (int)(((float)rs + 0.5f) * inv_s), j = rs - r * s.S + g.shift;
                const int rc = r * 4 + (j >> 1);
                if (it < items) b8[((rc * kStemBN + (k ^ (rc & 15))) << 1) + (j & 1)] = uint2{v[u].x, v[u].y};
            }
        }
    }

    const int npx = g.TH * TW;
    constexpr int BM = kSwCompute * 32;
    char* stage = reinterpret_cast<char*>(lds) + g.b_bytes + 2 * g.patch_bytes;
    const int c8 = lane & 7, l3 = lane >> 3;
    const size_t y_elems = (size_t)s.M * s.K;
    const int nblocks = t_end - t_begin;

    if (!computes) {
        // =========================== store waves ============================================
        // store wave sw carries fragments 2 sw and 2 sw + 1 (64 pixels), both filter halves
        const int sw = wave - kSwCompute;
        const uint32_t sr = stage_off(l3, c8);   // read-back: piece l%8 of pixel l/8 (+ 8j: 1024 bytes further on)
        const uint32_t y_lane = (uint32_t)(l3 * s.K + 4 * c8) * (uint32_t)sizeof(TO);
        bool k_ok[2];
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) k_ok[ni] = k0 + ni * 32 + 4 * c8 + 3 < s.K;
        __syncthreads();                        // weights and patch 0 are in LDS
        for (int it = 0; it <= nblocks; ++it) {
            u32x4 out[2][2][4];
            if (it > 0) {
#pragma unroll
                for (int f = 0; f < 2; ++f)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            out[f][ni][j] = *reinterpret_cast<const u32x4*>(stage + ((2 * sw + f) * 2 + ni) * 4096 + sr + j * 1024);
            }
            if (it < nblocks) __syncthreads();  // M: the area may be overwritten
            if (it > 0) {
                const StemTile tc = stem_decode(t_begin + it - 1, g);
                const size_t org = ((size_t)(tc.n * s.P + tc.p0) * s.Q + tc.q0) * s.K + k0;
                const size_t rem = (y_elems - org) * sizeof(TO);
                const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + org, 0, rem > 0xffffffffull ? 0xffffffffu : (uint32_t)rem,
                                                                       kRsrcFlags);
                const bool edge = npx < BM || tc.p0 + g.TH > s.P || tc.q0 + TW > s.Q;    // uniform
#pragma unroll
                for (int f = 0; f < 2; ++f)
#pragma unroll
                    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
                        for (int j = 0; j < 4; ++j) {
                            bool ok = k_ok[ni];
                            const int t0 = (2 * sw + f) * 32 + 8 * j;      // uniform
                            if (edge) {
                                const int t = t0 + l3;
                                ok = ok && t < npx && tc.p0 + (t >> g.TW_LOG2) < s.P && tc.q0 + (t & (TW - 1)) < s.Q;
                            }
                            const uint32_t y_uni = (uint32_t)(((t0 >> g.TW_LOG2) * s.Q + (t0 & (TW - 1))) * s.K + ni * 32) * (uint32_t)sizeof(TO);
                            if (ok) store_piece<TO>(out[f][ni][j], y_rsrc, y_lane + y_uni);
                        }
            }
            if (it < nblocks) __syncthreads();  // S: the next block's deposits are complete
        }
        return;
    }

    // =========================== compute waves ==============================================
    const int frow = lane & 31, fk = lane >> 5;
    const char* lds_b = reinterpret_cast<const char*>(lds);
    uint32_t a_off;                               // byte offset in the patch of the lane's run at filter row 0
    {
        const int t = wave * 32 + frow;
        const int th = t >> g.TW_LOG2, tw = t & (TW - 1);
        a_off = (uint32_t)(t < npx ? th * s.stride * g.PPAIRS + tw * (s.stride >> 1) + fk : fk) * 16u;
    }
    const uint32_t b_off = (uint32_t)(fk * kStemBN) * 16u;
    const uint32_t b_lane = (uint32_t)(frow ^ fk) * 16u;
    const uint32_t row_bytes = (uint32_t)g.PPAIRS * 16u;
    bool zero_lo[2], zero_hi[2];
#pragma unroll
    for (int kk = 0; kk < 2; ++kk) {
        const int j = 4 * kk + 2 * fk;
        zero_lo[kk] = j < g.shift || j >= s.S + g.shift;
        zero_hi[kk] = (j + 1) < g.shift || (j + 1) >= s.S + g.shift;
    }
    const bool mask_kk0 = g.shift != 0 || s.S + g.shift < 4;
    const bool mask_kk1 = s.S + g.shift < 8;
    char* stg = stage + wave * 2 * 4096;
    uint32_t sw_off[4];                           // deposit offset per filter quad
#pragma unroll
    for (int gq = 0; gq < 4; ++gq) sw_off[gq] = stage_off(frow, 2 * gq + fk);

    park_patch(0, pregs);
    // The patch of block b + 2 is requested in tick b and parked at the end of tick b + 1: a whole tick for the
    // loads, which queue behind the store waves' stores.  Two register sets that swap roles every tick.
    u32x4 pregs2[kSwPatchItems];
    if (t_begin + 1 < t_end) load_patch(t_begin + 1, pregs);
    __syncthreads();                            // weights and patch 0 are in LDS
    auto tick = [&](int tile, u32x4 (&pcur)[kSwPatchItems], u32x4 (&pnxt)[kSwPatchItems]) __attribute__((always_inline)) {
        const char* pa = lds_b + g.b_bytes + ((tile - t_begin) & 1) * g.patch_bytes;
        const char* pb = lds_b + b_off;
        floatx16 acc[2];
        frag_t a0, b0[2], a1, b1[2];

        auto fetch = [&](int r, int kk, frag_t& af, frag_t (&bf)[2]) {
            af = *reinterpret_cast<const frag_t*>(pa + a_off + (uint32_t)r * row_bytes + kk * 32);
#pragma unroll
            for (int ni = 0; ni < 2; ++ni)
                bf[ni] = *reinterpret_cast<const frag_t*>(pb + (b_lane ^ (uint32_t)(((4 * r + 2 * kk) & 15) << 4)) + r * 4096 +
                                                          kk * 2048 + ni * 512);
        };
        auto mma = [&](frag_t& af, frag_t (&bf)[2], int kk, bool first) {
            if (kk == 0 ? mask_kk0 : mask_kk1) {
                u32x4 v = __builtin_bit_cast(u32x4, af);
                if (zero_lo[kk]) { v.x = 0u; v.y = 0u; }
                if (zero_hi[kk]) { v.z = 0u; v.w = 0u; }
                af = __builtin_bit_cast(frag_t, v);
            }
#pragma unroll
            for (int ni = 0; ni < 2; ++ni) {
                if (first) {
                    floatx16 z;
#pragma unroll
                    for (int v = 0; v < 16; ++v) z[v] = 0.f;
                    acc[ni] = Elem<T>::mfma32(bf[ni], af, z);
                } else {
                    acc[ni] = Elem<T>::mfma32(bf[ni], af, acc[ni]);
                }
            }
        };
        const int r_last = s.R - 1;
        fetch(0, 0, a0, b0);
        fetch(0, 1, a1, b1);
        mma(a0, b0, 0, true);
        fetch(min(1, r_last), 0, a0, b0);
        mma(a1, b1, 1, false);
        // M after the first filter row: by now the store waves hold the previous block in registers, so neither
        // side waits long
        __syncthreads();
        if (tile + 2 < t_end) load_patch(tile + 2, pnxt);
        for (int r = 1; r < s.R; ++r) {
            fetch(r, 1, a1, b1);
            mma(a0, b0, 0, false);
            fetch(min(r + 1, r_last), 0, a0, b0);
            mma(a1, b1, 1, false);
        }
        // deposit: lane l holds block pixel 32*wave + l%32 and, in accumulator element v, filter
        // 8*(v/4) + 4*(l/32) + v%4 of the 32-wide half
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                u32x4 v;
                v.x = __float_as_uint(acc[ni][4 * gq]);     v.y = __float_as_uint(acc[ni][4 * gq + 1]);
                v.z = __float_as_uint(acc[ni][4 * gq + 2]); v.w = __float_as_uint(acc[ni][4 * gq + 3]);
                *reinterpret_cast<u32x4*>(stg + ni * 4096 + sw_off[gq]) = v;
            }
        if (tile + 1 < t_end) park_patch((tile + 1 - t_begin) & 1, pcur);
        __syncthreads();                        // S: deposits complete, next patch in LDS
    };
    for (int tile = t_begin; tile < t_end; tile += 2) {
        tick(tile, pregs, pregs2);
        if (tile + 1 < t_end) tick(tile + 1, pregs2, pregs);
    }
}

constexpr int kStemMI = 2;                       // 4 waves x 2 fragments x 32 = 256 output pixels per block
constexpr int kStemLdsLimit = 80 * 1024;     // two workgroups per compute unit
constexpr int kStemStageBytes = kStemWaves * 4096;

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
    const int ppairs_used = ((TW - 1) * s.stride + 8) / 2;
    // A fragment of 32 pixels is two block rows when TW = 16.  Its operand read is free of bank conflicts
    // when the second row starts a multiple of 16 pairs (256 bytes) after the first: the two halves of a
    // 16-lane pass (columns 0-3, 12-15 of one row, 4-11 of the other) then share a bank window without
    // overlapping.  Block rows are `stride` patch rows apart, so the pitch is padded to a multiple of 8.
    const int ppairs = tw_log2 == 4 ? (ppairs_used + 7) / 8 * 8 : ppairs_used;
    const long patch_bytes = (((long)PH * ppairs + 255) / 256) * 4096;   // whole workgroup-wide pieces
    if (patch_bytes > kStemPatchItems * 4096) return false;
    const long b_bytes = (long)s.R * 4 * kStemBN * 16;
    if (2 * patch_bytes + b_bytes + kStemStageBytes > kStemLdsLimit) return false;
    if ((long)TH * s.Q * s.K * 4 >= (1L << 31)) return false;            // in-block output offsets are 32-bit
    g->TH = TH; g->TW_LOG2 = tw_log2; g->PH = PH; g->PPAIRS = ppairs; g->PPAIRS_USED = ppairs_used;
    g->tiles_h = (s.P + TH - 1) / TH; g->tiles_w = (s.Q + TW - 1) / TW; g->tiles_n = (s.K + kStemBN - 1) / kStemBN;
    g->shift = shift; g->b_bytes = (int)b_bytes; g->patch_bytes = (int)patch_bytes; g->inv_ppairs = 1.0f / (float)ppairs;
    const long total = (long)s.N * g->tiles_h * g->tiles_w * g->tiles_n;
    if (total > 0x7fffffffL) return false;
    g->total_tiles = (int)total;
    return true;
}

constexpr int kSwLdsLimit = 160 * 1024;      // one workgroup per compute unit

// The form with store waves needs whole 16-byte pieces of y rows, one filter tile, and its staging area in LDS.
bool stem_sw_fits(const ConvShape& s, const StemGeom& g) {
    return g.tiles_n == 1 && (s.K & 3) == 0 && g.b_bytes + 2 * g.patch_bytes + kSwStageBytes <= kSwLdsLimit;
}

template <typename T, typename TO>
hipError_t launch_stem_sw_t(const void* x, const void* w, void* y, const ConvShape& s, StemGeom g, hipStream_t st) {
    const int lds_bytes = g.b_bytes + 2 * g.patch_bytes + kSwStageBytes;
    auto kern = stem_sw_kernel<T, TO>;
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kSwLdsLimit);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    // one workgroup per compute unit, each with an equal range of blocks
    const int cap = call_max_workgroups();
    const long slots = cap > 0 ? cap : (long)device_cus();
    const int nwg = (int)(g.total_tiles < slots ? g.total_tiles : slots);
    g.tiles_base = g.total_tiles / nwg;
    g.tiles_rem = g.total_tiles % nwg;
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kSwWaves * 64), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y, s, g);
    return hipGetLastError();
}

template <typename T, typename TO>
hipError_t launch_stem_t(const void* x, const void* w, void* y, const ConvShape& s, StemGeom g, hipStream_t st) {
    const int lds_bytes = g.b_bytes + 2 * g.patch_bytes + kStemStageBytes;
    auto kern = stem_kernel<T, TO, kStemMI>;
    const int threads = kStemWaves * 64;
    int nwg = g.total_tiles;
    // more than 64 KiB of dynamic LDS must be allowed once per kernel and process; a failed
    // attempt is retried by the next call
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kStemLdsLimit);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    if (g.tiles_n == 1) {
        // one filter tile: workgroups own ranges of blocks and keep the weights resident
        static std::atomic<long long> occ_slot{-1};
        const int occ = cached_occupancy(occ_slot, (const void*)kern, threads, lds_bytes);
        // The kernel waits on memory most of the time, so every workgroup slot of the device is
        // filled (as many resident workgroups per compute unit as fit), each with an equal range.
        const int cap = call_max_workgroups();
        const long slots = cap > 0 ? cap : (long)device_cus() * occ;
        const long per = (g.total_tiles + slots - 1) / slots;
        nwg = (int)((g.total_tiles + per - 1) / per);
    }
    g.tiles_base = g.total_tiles / nwg;
    g.tiles_rem = g.total_tiles % nwg;
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(threads), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y, s, g);
    return hipGetLastError();
}

}  // namespace

bool stem_supported(const ConvShape& s) {
    StemGeom g;
    return plan_stem(s, &g);
}

// Two forms: 0 = four waves that load, multiply and store, two workgroups per compute unit; 1 = eight compute
// and four store waves, one workgroup per compute unit.
int stem_num_variants() { return 2; }
const char* stem_variant_name(int v) { return v == 1 ? "stem_8+4" : "stem"; }
bool stem_variant_supported(const ConvShape& s, int v) {
    StemGeom g;
    if (!plan_stem(s, &g)) return false;
    return v == 0 || (v == 1 && stem_sw_fits(s, g));
}
// The form with store waves is the faster one (-7 to -15 % from two blocks per compute unit on, -10 % with at most one
// block per compute unit) except between one and two blocks per compute unit, where half of its workgroups have
// two blocks and the others wait (1.5 blocks per compute unit: +6 %).
int stem_choose(const ConvShape& s) {
    StemGeom g;
    if (!plan_stem(s, &g)) return -1;
    const long cus = device_cus();
    return stem_sw_fits(s, g) && (g.total_tiles <= cus || g.total_tiles >= 2 * cus) ? 1 : 0;
}

hipError_t launch_stem(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v, hipStream_t st) {
    StemGeom g;
    if (!plan_stem(s, &g)) return hipErrorInvalidConfiguration;
    if (v < 0 || v >= stem_num_variants() || !stem_variant_supported(s, v)) v = stem_choose(s);
    if (v == 1) {
        if (in_t == IN_BF16) {
            if (out_t == OUT_F32) return launch_stem_sw_t<bf16_t, float>(x, w, y, s, g, st);
            return launch_stem_sw_t<bf16_t, bf16_t>(x, w, y, s, g, st);
        }
        if (out_t == OUT_F32) return launch_stem_sw_t<f16_t, float>(x, w, y, s, g, st);
        return launch_stem_sw_t<f16_t, f16_t>(x, w, y, s, g, st);
    }
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_stem_t<bf16_t, float>(x, w, y, s, g, st);
        return launch_stem_t<bf16_t, bf16_t>(x, w, y, s, g, st);
    }
    if (out_t == OUT_F32) return launch_stem_t<f16_t, float>(x, w, y, s, g, st);
    return launch_stem_t<f16_t, f16_t>(x, w, y, s, g, st);
}

}  // namespace iconv

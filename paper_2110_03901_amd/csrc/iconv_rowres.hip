// Implicit channel-first im2col with inter-tile reuse (paper section 5), resident filters, for
// layers whose pixels are one or two 64-byte half-lines wide (C = 32 or 64): the row-phased
// resident-filter kernel.
//
// As in iconv_resident.hip the filters of 64 output channels and the input patch of an output
// block live in LDS and the K loop reads every operand from there (tap (r, s) of pixel (th, tw) is
// patch pixel (th*stride + r*dil, tw*stride + s*dil), a channel-contiguous run as in section 3.1).
// What differs is how the block reaches LDS and when the matrix cores may start:
//
//  * An LDS row is a WHOLE pixel (all C channels, 2*C bytes) or a whole filter tap, so one
//    global -> LDS load instruction fetches complete 128-byte lines (8 pixels, or 8 filters of a
//    tap, per instruction at C = 64).  Slicing the channels instead -- 64 bytes of each pixel per
//    load -- touches every line of x twice, and timestamps showed the front end of the memory pipe
//    (lines touched per instruction), not bytes, to bound the 2.8 us before the first MFMA.
//  * The work of a block is phased by FILTER ROW r (the decomposed 1x1 convolutions of section 3.2
//    in their natural order): phase r needs the R-th part of the filters and the patch rows up to
//    r*dil + (TH-1)*stride only, i.e. phase 0 waits for 88 of the 152 KB of a 56-wide 3x3, 64-channel
//    block, and rows and taps of later phases land under the MFMAs of earlier ones.
//  * Everything a wave needs before its first load is a handful of scalar operations: lane offsets are
//    two adds and a mask test per load, out-of-image pixels are a per-lane bit mask over the pixel
//    groups of a patch row.
//
// Waves: four compute waves (pixel half x filter half, MF accumulator tiles of 32x32, as in
// iconv_resident.hip) and four loader waves, persistent over a range of blocks (the next block is
// loaded under the stores of the current one) -- or, for launches with one block per workgroup
// (SPLIT), eight waves that all compute: the four that issue the later phases take the last MF/2
// fragments of their (pixel half, filter half), so that every SIMD has two waves issuing MFMAs and
// each hides the other's operand reads and address arithmetic (19-20 ns -> about 17.5 ns per MFMA).
// LDS: [filters: tap x 64 filters x 2C bytes]
// [patch: PH rows x PWp pixels x 2C bytes][staging: 2 KiB per compute wave].  Chunk c (16 bytes) of
// row i is stored at chunk  c ^ swz(i),  swz(i) = (i >> 1) & 7 for 128-byte rows, (i >> 2) & 3 for
// 64-byte rows: the 16 lanes the LDS serves in one pass of a ds_read_b128 (lanes 0-3, 12-15, 20-27 or
// 4-11, 16-19, 28-31 of a half-wave) then hit 16 different 16-byte slots of the 256-byte bank window
// when their rows are consecutive.  The 32 pixels of a fragment are consecutive in the OUTPUT block;
// where they run on into the next block row their patch pixels jump by PWp - TW, which for
// TW = 8 (mod 16) is exactly the top bit of the swizzle term: odd patch rows are therefore stored with
// that bit flipped ("skew"), which makes the term the one the pixel would have in a patch with rows
// of TW pixels.  Filter row r reads patch rows r*dil further down; for odd r*dil the flip merges
// with the K-step bits of the address, so it costs nothing in the loop.
#include <atomic>
#include <type_traits>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

constexpr int kRowWaves = 4;         // compute waves
constexpr int kRowLoaders = 4;       // loader waves
constexpr int kRowBN = 64;           // filters per workgroup (filter rows in LDS; rows beyond K read as zeros)
constexpr int kRowStage = 2048;      // output staging bytes per compute wave
constexpr int kRowMaxR = 8;          // filter rows (phases per block) the wait bookkeeping holds

struct RowGeom {
    int TH, TW;          // output block
    int PH, PWp;         // input patch rows; pixels per patch row in LDS (multiple of 16)
    int tiles_h, tiles_w;
    int total_tiles;
    int tiles_base, tiles_rem;   // workgroup i owns tiles_base (+1 if i < tiles_rem) consecutive blocks
    int w_bytes;         // LDS bytes of the filters: R*S*64 rows
    int patch_bytes;     // LDS bytes of the patch
    int rows0;           // patch rows phase 0 needs: (TH-1)*stride + 1
    int skew;            // 1: odd patch rows are stored with the top swizzle bit flipped
    float inv_tw, inv_tiles_w, inv_tiles_h;
};

struct RowTile {
    int n, p0, q0;
};

// (float reciprocals instead of integer division: exact for the block counts the planner allows)
__device__ __forceinline__ RowTile row_decode(int t, const RowGeom& g) {
    RowTile c;
    int tile_w = 0, rest = t;
    if (g.tiles_w > 1) {
        rest = (int)(((float)t + 0.5f) * g.inv_tiles_w);
        tile_w = t - rest * g.tiles_w;
    }
    c.n = (int)(((float)rest + 0.5f) * g.inv_tiles_h);
    const int tile_h = rest - c.n * g.tiles_h;
    c.p0 = tile_h * g.TH; c.q0 = tile_w * g.TW;
    return c;
}

__device__ __forceinline__ void wait_vmcnt_upto(int n) {
    switch (n) {
#define ICONV_W(k) case k: wait_vmcnt<k>(); break;
        ICONV_W(0) ICONV_W(1) ICONV_W(2) ICONV_W(3) ICONV_W(4) ICONV_W(5) ICONV_W(6) ICONV_W(7)
        ICONV_W(8) ICONV_W(9) ICONV_W(10) ICONV_W(11) ICONV_W(12) ICONV_W(13) ICONV_W(14) ICONV_W(15)
        ICONV_W(16) ICONV_W(17) ICONV_W(18) ICONV_W(19) ICONV_W(20) ICONV_W(21) ICONV_W(22) ICONV_W(23)
        ICONV_W(24) ICONV_W(25) ICONV_W(26) ICONV_W(27) ICONV_W(28) ICONV_W(29) ICONV_W(30) ICONV_W(31)
        ICONV_W(32) ICONV_W(33) ICONV_W(34) ICONV_W(35) ICONV_W(36) ICONV_W(37) ICONV_W(38) ICONV_W(39)
        ICONV_W(40) ICONV_W(41) ICONV_W(42) ICONV_W(43) ICONV_W(44) ICONV_W(45) ICONV_W(46) ICONV_W(47)
        ICONV_W(48) ICONV_W(49) ICONV_W(50) ICONV_W(51) ICONV_W(52) ICONV_W(53) ICONV_W(54) ICONV_W(55)
#undef ICONV_W
        default: wait_vmcnt<0>(); break;
    }
}

template <int V> using IC = std::integral_constant<int, V>;    // a fragment index as a type

template <typename T, typename TO, int MF, int S_, int CPR, int SPLIT>
__global__ void __launch_bounds__((kRowWaves + kRowLoaders) * 64)
irow_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const RowGeom g) {
    typedef typename Elem<T>::frag frag_t;
    constexpr int NWAVES = kRowWaves + kRowLoaders;
    constexpr int RB = CPR * 16;                // bytes of an LDS row (a pixel, or a filter tap)
    constexpr int PPL = 64 / CPR;               // rows one wave-wide load fills
    constexpr int KK = CPR / 2;                 // K steps of 16 channels per tap
    constexpr int SWB = CPR == 8 ? 3 : 2;       // bits of the swizzle term
    constexpr int SWS = CPR == 8 ? 1 : 2;       // swz(i) = (i >> SWS) & (CPR - 1)
    constexpr uint32_t kSkewBit = 16u << (SWB - 1);   // byte-address bit of the top swizzle bit
    constexpr int FG = kRowBN / PPL;            // filter groups (loads) per tap
    extern __shared__ u32x4 lds[];
    touch_kernargs<24 + sizeof(ConvShape) + sizeof(RowGeom)>();

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int t_begin = wg * g.tiles_base + min(wg, g.tiles_rem);
    const int nblocks = g.tiles_base + (wg < g.tiles_rem ? 1 : 0);
    if (nblocks <= 0) return;
    const int R = s.R;

    const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * s.C * 2u;
    const uint32_t w_bytes = (uint32_t)s.K * s.Kg * 2u;
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
    const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds;
    const uint32_t patch_base = lds_base + (uint32_t)g.w_bytes;

    // ---- loads.  A wave-wide load fills PPL consecutive LDS rows: lane l owns row l / CPR of the
    // group and physical chunk l % CPR, and fetches the logical chunk that is stored there.  Within a
    // group the swizzle term is the row-in-group part plus, for 128-byte rows, a bit that alternates
    // with the group number; both, and the skew of odd patch rows, are the same bit for all lanes of a
    // load, so a load's lane offsets are the lane's constant, a wave-uniform offset and a uniform flip.
    const int l_row = lane / CPR;
    const int l_chunk = (lane % CPR) ^ ((l_row >> SWS) & (CPR - 1));
    const uint32_t grp_flip_mask = CPR == 8 ? 1u : 0u;        // 128-byte rows: odd groups flip the top swizzle bit
    const uint32_t x_lane = (uint32_t)(l_row * s.C + l_chunk * 8) * 2u;
    const uint32_t w_lane = (uint32_t)(l_row * s.Kg + l_chunk * 8) * 2u;
    const uint32_t kOut = 0x80000000u;          // lane offset that reads zeros (tensors are smaller than 2^31 bytes + 2^31)
    const int groups = g.PWp / PPL;             // pixel groups per patch row (at most 32)

    // Loads of phase r of the block at (n, p0, q0), in one fixed order -- the S_*FG filter loads of
    // filter row r (skipped when the filters are already resident), then the patch rows the phase adds
    // -- of which this wave takes every nparts-th starting at `part`.  Returns the number issued.
    // per-lane validity of the lane's pixel column in each pixel group of a patch row (bit grp)
    auto column_mask = [&](const RowTile& tc) {
        const int w_org = tc.q0 * s.stride - s.pad;
        uint32_t m = 0;
        for (int gq = 0; gq < groups; ++gq) m |= ((unsigned)(w_org + gq * PPL + l_row) < (unsigned)s.W ? 1u : 0u) << gq;
        return m;
    };
    auto issue_phase = [&](const RowTile& tc, uint32_t col_ok, int r, int part, int nparts, bool with_filters) {
        int issued = 0;
        int j = part;
        if (with_filters) {
            for (; j < S_ * FG; j += nparts, ++issued) {
                const int sc = j / FG, fg = j - sc * FG;
                const uint32_t soff = (uint32_t)((r * S_ + sc) * s.C) * 2u + (uint32_t)(fg * PPL) * (uint32_t)s.Kg * 2u;
                const uint32_t flip = ((uint32_t)fg & grp_flip_mask) * kSkewBit;
                const bool ok = fg * PPL + l_row < s.K;
                dma16s(w_rsrc, ok ? (w_lane ^ flip) : kOut, soff,
                       (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + (uint32_t)(((r * S_ + sc) * FG + fg) * 1024))));
            }
            j -= S_ * FG;
        }
        const int row_lo = r == 0 ? 0 : min(g.PH, (r - 1) * s.dil + g.rows0);
        const int row_hi = min(g.PH, r * s.dil + g.rows0);
        const int count = (row_hi - row_lo) * groups;
        const int h_org = tc.p0 * s.stride - s.pad, w_org = tc.q0 * s.stride - s.pad;
        const uint32_t x_col = x_lane + (uint32_t)(w_org * s.C * 2);      // may wrap below zero: only where col_ok is clear
        int row = row_lo + j / groups, grp = j - (j / groups) * groups;
        const int drow = nparts / groups, dgrp = nparts - drow * groups;
        for (; j < count; j += nparts, ++issued) {
            const int h = h_org + row;
            const bool row_ok = (unsigned)h < (unsigned)s.H;                  // uniform
            const uint32_t soff = (uint32_t)((tc.n * s.H + (row_ok ? h : 0)) * s.W) * (uint32_t)s.C * 2u;
            const uint32_t flip = (((uint32_t)grp & grp_flip_mask) ^ (uint32_t)(g.skew & row & 1)) * kSkewBit;
            const bool ok = row_ok && ((col_ok >> grp) & 1u);
            const uint32_t voff = (x_col + (uint32_t)(grp * PPL * s.C * 2)) ^ flip;
            dma16s(x_rsrc, ok ? voff : kOut, soff,
                   (uint32_t)__builtin_amdgcn_readfirstlane((int)(patch_base + (uint32_t)((row * groups + grp) * 1024))));
            grp += dgrp; row += drow;
            if (grp >= groups) { grp -= groups; ++row; }
        }
        return issued;
    };

    // ---- first block: phase 0 is issued by all eight waves, later phases by the loader waves
    RowTile tc0 = row_decode(t_begin, g);
    int pending[kRowMaxR];                      // this wave's loads of phase r of the block being loaded
#pragma unroll
    for (int r = 0; r < kRowMaxR; ++r) pending[r] = 0;
    const uint32_t col_ok0 = column_mask(tc0);
    pending[0] = issue_phase(tc0, col_ok0, 0, wave, NWAVES, true);

    if (SPLIT == 0 && wave >= kRowWaves) {
        // =========================== loader waves ===========================================
        __builtin_amdgcn_s_setprio(3);
        const int lw = wave - kRowWaves;
        // First block: the loads of filter row r + 1 are issued once phase r has been handed over, so
        // that the wait for phase r is not held up by the issue of later loads (a load instruction
        // occupies its wave for about 0.1 us while the memory pipe is busy).  Later blocks: all phases
        // are issued at once, under the previous block's stores.
        bool first_block = true;
        for (int b = 0; b < nblocks; ++b) {
            int later = 0;
#pragma unroll
            for (int r = 0; r < kRowMaxR; ++r) later += pending[r];
#pragma unroll
            for (int r = 0; r < kRowMaxR; ++r) {
                if (r < R) {
                    later -= pending[r];
                    wait_vmcnt_upto(later);         // this wave's loads of phases 0 .. r have landed
                    __syncthreads();                // phase r of block b is in LDS
                    if (first_block && r + 1 < R) {
                        const int c = issue_phase(tc0, col_ok0, r + 1, lw, kRowLoaders, true);
                        if (r + 1 < kRowMaxR) pending[r + 1 < kRowMaxR ? r + 1 : 0] = c;
                        later += c;
                    }
                }
            }
            first_block = false;
            if (b + 1 < nblocks) {
                __syncthreads();                    // every compute wave has left the K loop of block b: the patch is free
                const RowTile tn = row_decode(t_begin + b + 1, g);
                const uint32_t col_ok = column_mask(tn);
#pragma unroll
                for (int r = 0; r < kRowMaxR; ++r) pending[r] = r < R ? issue_phase(tn, col_ok, r, lw, kRowLoaders, false) : 0;
            }
        }
        return;
    }

    // =============================== compute waves ==============================================
    // SPLIT == 0: waves 0-3 compute all MF fragments of their (pixel half, filter half).  SPLIT == 1 (one block per
    // workgroup): the four waves that issue the later phases compute as well -- waves 0-3 take fragments 0 .. MFA-1,
    // waves 4-7 issue phase r + 1 after barrier r and then take fragments MFA .. MF-1 -- so that every SIMD has two
    // waves with MFMAs to issue and one hides the other's operand reads and address arithmetic.
    constexpr int MFA = SPLIT ? (MF + 1) / 2 : MF;
    auto compute = [&](auto f0_t, auto nf_t, auto issues_t) {
        constexpr int F0 = decltype(f0_t)::value, NF = decltype(nf_t)::value;
        constexpr bool ISSUES = decltype(issues_t)::value;
        const int frow = lane & 31, fk = lane >> 5;
        const int wv = wave & 3;
        const int m_half = wv >> 1, nh = wv & 1;
        const int npx = g.TH * g.TW;
        const char* lds_b = reinterpret_cast<const char*>(lds);
        // Byte offset in the patch of the lane's operand of fragment mf, tap column s, filter row 0 and
        // K step 0: pixel (th*stride, tw*stride + s*dil), chunk l/32.  K step kk: chunk 2*kk + l/32, i.e. the
        // offset xor (kk << 5); a filter row further down adds a multiple of 16 rows, which leaves the
        // swizzle term alone apart from the skew bit.  So: one (a ^ mask) + row offset per operand read.
        uint32_t a_addr[NF][S_];
#pragma unroll
        for (int mf = 0; mf < NF; ++mf) {
            const int t = (m_half * MF + F0 + mf) * 32 + frow;
            const int th = (int)(((float)t + 0.5f) * g.inv_tw);
            const int tw = t - th * g.TW;
#pragma unroll
            for (int sc = 0; sc < S_; ++sc) {
                const int pix = t < npx ? (th * g.PWp + tw) * s.stride + sc * s.dil : sc * s.dil;
                const int odd_row = t < npx ? (g.skew & th & 1) << (SWB - 1) : 0;       // skew implies stride 1: patch row = th
                a_addr[mf][sc] = (uint32_t)(pix * RB + ((fk ^ ((pix >> SWS) & (CPR - 1)) ^ odd_row) << 4));
            }
        }
        const uint32_t row_step = (uint32_t)(s.dil * g.PWp * RB);
        // filter fragment of (tap, K step kk): filter f = 32*nh + l%32, chunk 2*kk + l/32
        const int f_lane = nh * 32 + frow;
        const uint32_t b_lane = (uint32_t)(f_lane * RB + ((fk ^ ((f_lane >> SWS) & (CPR - 1))) << 4));
        // output staging, 16 pixels x 32 filters at a time: piece c (16 bytes, 4 filters) of pixel i at
        // stage_off(i, c).  The waves that also load have no staging area of their own: they use the LDS rows of
        // filter row 0, which no wave reads after the barrier that opens filter row 1 (the host asks for R >= 2).
        char* stg = reinterpret_cast<char*>(lds) + (ISSUES ? wv * kRowStage : g.w_bytes + g.patch_bytes + wave * kRowStage);
        const int f16 = frow & 15;
        const uint32_t sw0 = stage_off(f16, fk);        // piece 2*gq + fk: xor (gq << 5)
        const int l8 = lane >> 3, c8 = lane & 7;
        const uint32_t sr0 = stage_off(l8, c8);          // pixel l/8 (+8), piece l%8
        const uint32_t sr1 = stage_off(l8 + 8, c8);
        const size_t y_elems = (size_t)s.M * s.K;
        const bool k_ok = nh * 32 + 4 * c8 + 3 < s.K;

        floatx16 acc[NF];

        // ---- the K loop of filter row r: K steps (s, kk) = (0,0) .. (0,KK-1), (1,0), ...  In every step
        // the filter fragment of the next step is read into the other B register set first, and each pixel
        // fragment is re-read for the next step as soon as its MFMA has been issued, so the LDS reads of a
        // step run under the MFMAs of the step before.
        auto fetch_a = [&](int mf, int sc, uint32_t mask, uint32_t roff_v) {
            uint32_t addr;
            asm volatile("v_xad_u32 %0, %1, %2, %3" : "=v"(addr) : "v"(a_addr[mf][sc]), "s"(mask), "v"(roff_v));
            return *reinterpret_cast<const frag_t __attribute__((address_space(3)))*>(addr);
        };
        auto fetch_b = [&](int tap, int kk) {
            return *reinterpret_cast<const frag_t*>(lds_b + tap * (kRowBN * RB) + (b_lane ^ (uint32_t)(kk << 5)));
        };
        auto flipped = [&](int r) { return (uint32_t)(g.skew & (r * s.dil) & 1) * kSkewBit; };
        frag_t af[NF], b0, b1;
        auto row = [&](int r, auto first, auto lo_t, auto hi_t) {
            constexpr int LO = decltype(lo_t)::value, HI = decltype(hi_t)::value;
            uint32_t roff = patch_base + (uint32_t)r * row_step;
            asm volatile("" : "+v"(roff));          // one copy in a vector register for the whole row
            const uint32_t mask_c = flipped(r);
            // the row's first operands
            b0 = fetch_b(r * S_, 0);
#pragma unroll
            for (int mf = LO; mf < HI; ++mf) af[mf] = fetch_a(mf, 0, mask_c, roff);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int st = 0; st < KK * S_; ++st) {
                const bool last = st + 1 == KK * S_;
                const int sc_n = last ? 0 : (st + 1) / KK, kk_n = last ? 0 : (st + 1) % KK;
                frag_t& bc = (st & 1) ? b1 : b0;
                frag_t& bn = (st & 1) ? b0 : b1;
                if (!last) bn = fetch_b(r * S_ + sc_n, kk_n);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mf = LO; mf < HI; ++mf) {
                    if (decltype(first)::value && st == 0) {
                        floatx16 z;
#pragma unroll
                        for (int v = 0; v < 16; ++v) z[v] = 0.f;
                        acc[mf] = Elem<T>::mfma32(bc, af[mf], z);
                    } else {
                        acc[mf] = Elem<T>::mfma32(bc, af[mf], acc[mf]);
                    }
                    if (!last) af[mf] = fetch_a(mf, sc_n, mask_c ^ (uint32_t)(kk_n << 5), roff);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };

        // ---- the epilogue of a block.  The filters are the MFMA's row operand: lane l holds pixel l%32 of
        // fragment mf and, in accumulator element v, filter 32*nh + 8*(v/4) + 4*(l/32) + v%4.  Half a
        // fragment (16 pixels x 32 filters) at a time goes through the wave's staging area (in-order LDS,
        // no wait needed in between) and leaves as 16-byte pieces, 8 lanes per pixel = one 128-byte line.
        auto epilogue = [&](const RowTile& tc, auto lo_t, auto hi_t) {
            constexpr int LO = decltype(lo_t)::value, HI = decltype(hi_t)::value;
            const size_t org = ((size_t)(tc.n * s.P + tc.p0) * s.Q + tc.q0) * s.K;
            const size_t rem = (y_elems - org) * sizeof(TO);
            const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + org, 0, rem > 0xffffffffull ? 0xffffffffu : (uint32_t)rem,
                                                                   kRsrcFlags);
            int l8v = l8;
            asm volatile("" : "+v"(l8v));           // the pixel arithmetic below is redone per block, not kept across the K loop
#pragma unroll
            for (int mf = LO; mf < HI; ++mf) {
                u32x4 out[2][2];
#pragma unroll
                for (int h = 0; h < 2; ++h) {
                    __builtin_amdgcn_wave_barrier();
                    if ((frow >> 4) == h) {
#pragma unroll
                        for (int gq = 0; gq < 4; ++gq) {
                            floatx4 v = {acc[mf][4 * gq], acc[mf][4 * gq + 1], acc[mf][4 * gq + 2], acc[mf][4 * gq + 3]};
                            *reinterpret_cast<floatx4*>(stg + (sw0 ^ (uint32_t)(gq << 5))) = v;
                        }
                    }
                    __builtin_amdgcn_wave_barrier();
                    out[h][0] = *reinterpret_cast<const u32x4*>(stg + sr0);
                    out[h][1] = *reinterpret_cast<const u32x4*>(stg + sr1);
                }
#pragma unroll
                for (int h = 0; h < 2; ++h)
#pragma unroll
                    for (int j = 0; j < 2; ++j) {
                        const int t = (m_half * MF + F0 + mf) * 32 + h * 16 + 8 * j + l8v;
                        const int th = (int)(((float)t + 0.5f) * g.inv_tw);
                        const int tw = t - th * g.TW;
                        const bool ok = k_ok & (t < npx) & (tc.p0 + th < s.P) & (tc.q0 + tw < s.Q);
                        const uint32_t off = (uint32_t)((th * s.Q + tw) * s.K + nh * 32 + 4 * c8) * (uint32_t)sizeof(TO);
                        if (ok) store_piece<TO>(out[h][j], y_rsrc, off);
                    }
            }
        };

        if constexpr (SPLIT == 0) {
            wait_vmcnt<0>();                        // this wave's share of the first block's phase 0
            for (int b = 0; b < nblocks; ++b) {
                __syncthreads();                    // filter row 0 and its patch rows are in LDS
                row(0, std::true_type{}, IC<0>{}, IC<NF>{});
                for (int r = 1; r < R; ++r) {
                    __syncthreads();                // filter row r and the patch rows it adds are in LDS
                    row(r, std::false_type{}, IC<0>{}, IC<NF>{});
                }
                if (b + 1 < nblocks) __syncthreads();   // the patch may be overwritten
                epilogue(b == 0 ? tc0 : row_decode(t_begin + b, g), IC<0>{}, IC<NF>{});
            }
        } else {
            // one block: every wave waits for its own loads of the phase, the barrier makes the phase complete,
            // and the waves that load issue the next phase before they start on the row
            int in_flight = 0;
            for (int r = 0; r + 1 < R; ++r) {
                wait_vmcnt<0>();
                __syncthreads();                    // filter row r and the patch rows it adds are in LDS
                if (ISSUES && r + 1 < R) in_flight = issue_phase(tc0, col_ok0, r + 1, wv, kRowLoaders, true);
                if (r == 0) row(0, std::true_type{}, IC<0>{}, IC<NF>{});
                else row(r, std::false_type{}, IC<0>{}, IC<NF>{});
            }
            (void)in_flight;
            wait_vmcnt<0>();
            __syncthreads();
            // The last filter row in groups of two fragments: a group's stores run under the next group's MFMAs (the
            // filter fragments are read once more per group).  Measured: -2...3 % at 24-32 images, no change at 16;
            // groups of one fragment are better at 32 images but 2 % worse at 16.
            constexpr int GS = 2;
            auto grp = [&](auto lo_t) {
                constexpr int LO = decltype(lo_t)::value;
                constexpr int HI = LO + GS < NF ? LO + GS : NF;
                if constexpr (LO < NF) {
                    row(R - 1, std::false_type{}, IC<LO>{}, IC<HI>{});
                    epilogue(tc0, IC<LO>{}, IC<HI>{});
                }
            };
            grp(IC<0>{}); grp(IC<GS>{}); grp(IC<2 * GS>{}); grp(IC<3 * GS>{});
        }
    };
    if constexpr (SPLIT == 0) {
        compute(IC<0>{}, IC<MF>{}, std::false_type{});
    } else {
        if (wave < kRowWaves) compute(IC<0>{}, IC<MFA>{}, std::false_type{});
        else compute(IC<MFA>{}, IC<MF - MFA>{}, std::true_type{});
    }
}


constexpr int kRowLdsLimit = 160 * 1024;

// Chooses the output block TH x TW (TH*TW <= 64*MF) for a fragment count MF; cost model as for the
// other patch kernels: MFMA work of all (padded) blocks plus the patch pixels brought into LDS.
bool plan_row(const ConvShape& s, int MF, RowGeom* g, double* cost_out) {
    if (s.C != 32 && s.C != 64) return false;
    if ((s.K & 3) != 0 || s.K > kRowBN || s.R > kRowMaxR) return false;
    if (s.S != 1 && s.S != 3) return false;                    // the filter width is a compile-time parameter
    if (MF == 8 && s.S == 3) return false;                     // eight fragments and three address sets exceed the register file
    if ((long long)s.N * s.H * s.W * s.C * 2 >= (1LL << 31)) return false;   // the zero-fill marker needs the upper half of the offsets
    const int RB = s.C * 2, PPL = 1024 / RB;
    const int BM = 2 * MF * 32;
    const int RS = s.R * s.S;
    const long w_lds = (long)RS * kRowBN * RB;
    double best = 1e300;
    bool found = false;
    for (int tw = 1; tw <= s.Q && tw <= BM; ++tw) {
        int th = BM / tw;
        if (th > s.P) th = s.P;
        if (th < 1) continue;
        const int ph = (th - 1) * s.stride + (s.R - 1) * s.dil + 1;
        const int pw = (tw - 1) * s.stride + (s.S - 1) * s.dil + 1;
        const int pwp = (pw + 15) & ~15;
        const long patch = (long)ph * pwp * RB;
        if (w_lds + patch + kRowWaves * kRowStage > kRowLdsLimit) continue;
        if (pwp / PPL > 32) continue;                                      // the column mask has one bit per pixel group
        if ((long)th * s.Q * s.K * 4 >= (1L << 31)) continue;             // in-block output offsets are 32-bit
        const long tiles = (long)((s.P + th - 1) / th) * ((s.Q + tw - 1) / tw);
        const double cost = (double)tiles * ((double)BM * RS + 4.0 * (double)ph * pwp);
        if (cost < best) {
            best = cost;
            found = true;
            g->TH = th; g->TW = tw; g->PH = ph; g->PWp = pwp;
            g->tiles_h = (s.P + th - 1) / th; g->tiles_w = (s.Q + tw - 1) / tw;
            g->w_bytes = (int)w_lds; g->patch_bytes = (int)patch;
            g->rows0 = (th - 1) * s.stride + 1;
            g->skew = (s.stride == 1 && (tw & 15) == 8) ? 1 : 0;
            g->inv_tw = 1.0f / (float)tw;
            g->inv_tiles_w = 1.0f / (float)g->tiles_w; g->inv_tiles_h = 1.0f / (float)g->tiles_h;
        }
    }
    if (!found) return false;
    const long total = (long)s.N * g->tiles_h * g->tiles_w;
    if (total >= (1L << 22)) return false;                     // block numbers are decoded with float reciprocals
    g->total_tiles = (int)total;
    if (cost_out) *cost_out = best * (double)s.N;
    return true;
}

template <typename T, typename TO, int MF, int S_, int CPR, int SPLIT>
hipError_t launch_row_t(const void* x, const void* w, void* y, const ConvShape& s, RowGeom g, hipStream_t st) {
    const int lds_bytes = g.w_bytes + g.patch_bytes + kRowWaves * kRowStage;
    auto kern = irow_kernel<T, TO, MF, S_, CPR, SPLIT>;
    const int threads = (kRowWaves + kRowLoaders) * 64;
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kRowLdsLimit);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    int nwg;
    if (SPLIT) {
        nwg = g.total_tiles;                    // one block per workgroup: all eight waves compute, nothing is left to prefetch
    } else {
        static std::atomic<long long> occ_slot{-1};
        const int occ = cached_occupancy(occ_slot, (const void*)kern, threads, lds_bytes);
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

template <int MF, int S_, int CPR, int SPLIT>
hipError_t launch_row_types(const void* x, const void* w, void* y, const ConvShape& s, const RowGeom& g, int in_t, int out_t,
                            hipStream_t st) {
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_row_t<bf16_t, float, MF, S_, CPR, SPLIT>(x, w, y, s, g, st);
        return launch_row_t<bf16_t, bf16_t, MF, S_, CPR, SPLIT>(x, w, y, s, g, st);
    }
    if (out_t == OUT_F32) return launch_row_t<f16_t, float, MF, S_, CPR, SPLIT>(x, w, y, s, g, st);
    return launch_row_t<f16_t, f16_t, MF, S_, CPR, SPLIT>(x, w, y, s, g, st);
}

template <int MF, int SPLIT>
hipError_t launch_row_mf(const void* x, const void* w, void* y, const ConvShape& s, const RowGeom& g, int in_t, int out_t,
                         hipStream_t st) {
    if (s.C == 64) {
        if (s.S == 1) return launch_row_types<MF, 1, 8, SPLIT>(x, w, y, s, g, in_t, out_t, st);
        return launch_row_types<MF, 3, 8, SPLIT>(x, w, y, s, g, in_t, out_t, st);
    }
    if (s.S == 1) return launch_row_types<MF, 1, 4, SPLIT>(x, w, y, s, g, in_t, out_t, st);
    return launch_row_types<MF, 3, 4, SPLIT>(x, w, y, s, g, in_t, out_t, st);
}

constexpr int kRowMF[] = {7, 8, 7, 8};      // variants 0, 1: four compute + four loader waves; 2, 3: all eight compute

// the all-compute form handles one block per workgroup and stages half of its output in the LDS rows of filter row 0
bool plan_variant(const ConvShape& s, int v, RowGeom* g, double* cost) {
    if (v < 0 || v >= 4 || !plan_row(s, kRowMF[v], g, cost)) return false;
    return v < 2 || s.R >= 2;
}

}  // namespace

bool rowres_supported(const ConvShape& s, int v) {
    RowGeom g;
    return plan_variant(s, v, &g, nullptr);
}

bool rowres_plan_cost(const ConvShape& s, int v, double* cost, long* blocks) {
    RowGeom g;
    if (!plan_variant(s, v, &g, cost)) return false;
    *blocks = g.total_tiles;
    return true;
}

hipError_t launch_rowres(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v, hipStream_t st) {
    RowGeom g;
    if (!plan_variant(s, v, &g, nullptr)) return hipErrorInvalidConfiguration;
    switch (v) {
        case 0: return launch_row_mf<7, 0>(x, w, y, s, g, in_t, out_t, st);
        case 1: return launch_row_mf<8, 0>(x, w, y, s, g, in_t, out_t, st);
        case 2: return launch_row_mf<7, 1>(x, w, y, s, g, in_t, out_t, st);
        default: return launch_row_mf<8, 1>(x, w, y, s, g, in_t, out_t, st);
    }
}

}  // namespace iconv

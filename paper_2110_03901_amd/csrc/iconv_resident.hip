// Implicit channel-first im2col with inter-tile reuse (paper section 5) for layers whose whole
// filter tensor slice fits on chip: the resident-filter kernel.
//
// For the early layers of a network (few channels, few filters) the filters of 64 output
// channels take R*S*C*128 bytes -- 72 KiB for a 3x3 layer with 64 channels -- and the input
// footprint of a few hundred output pixels about as much.  Both are placed in LDS ONCE per
// output block: the K loop (channel slice of 32 outer, tap (r, s) inner, the order of the
// paper's reuse scheme) then runs without any further global traffic and with a single barrier
// per channel slice, and the A operand of pixel (th, tw) and tap (r, s) is patch pixel
// (th*stride + r*dil, tw*stride + s*dil), a channel-contiguous run exactly as in section 3.1.
// The filters stay for all blocks of a persistent workgroup.
//
// Waves.  Four compute waves (one per SIMD): wave w owns pixel half w/2 of the block (MF fragments
// of 32 pixels) and filter half w%2 (32 filters), i.e. MF accumulator tiles of the 32x32x16 MFMA,
// the instruction a single wave per SIMD can issue at full rate.  One K step of 16 channels reads
// MF pixel fragments and one filter fragment for MF MFMAs.  Blocks of 64*MF pixels tile feature
// maps whose width is a multiple of 7 (MF = 7) or 8 without padding rows of the MFMA.  Four loader
// waves issue the global -> LDS loads: at the start those of the first NR phases (a phase is one
// channel slice of one block; NR patch regions exist), the first phase's with the help of the
// compute waves; afterwards, each time a phase has been computed, those of the phase that
// reuses its region, so loading, computing and the previous block's stores overlap.
//
// LDS.  Patch slice and filter slice use the same layout: rows (a pixel, or a filter) of 64
// bytes = four 16-byte chunks of 8 channels, chunk c of row i stored at chunk c ^ ((i >> 2) & 3);
// patch rows are padded to a multiple of 16 pixels.
// A ds_read_b128 is served in four passes of 16 lanes (lanes 0-3, 12-15, 20-27 / 4-11, 16-19,
// 28-31 of each half-wave, as measured on this chip), and a pass is conflict-free when its 16
// lanes fall on 16 different 16-byte positions of the 256-byte bank window.  With pixels that
// are consecutive in LDS the layout above achieves that.  The 32 pixels of a fragment are
// consecutive in the OUTPUT block, though: where they run from one block row into the next,
// their patch pixels jump by PWp - TW, which shifts the swizzle term and makes two lane groups of
// a pass collide (three of seven fragments for 56-wide rows in 64-pixel patch rows).  When
// TW = 8 (mod 16) at stride 1 the jump is 8 (mod 16) pixels, i.e. exactly bit 1 of the swizzle
// term, and storing ODD patch rows with bit 1 of the chunk number flipped ("skew") cancels it:
// the term then is the one the pixel would have in a patch with rows of TW pixels, where the
// fragment's pixels ARE consecutive.  A filter row r reads patch rows r*dil further down, so for
// odd r*dil the flip coincides with the K-step bit (chunk 2*kk + l/32) and costs nothing.
#include <atomic>
#include <type_traits>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

constexpr int kResWaves = 4;         // compute waves
constexpr int kResLoaders = 4;       // loader waves
constexpr int kResBN = 64;           // filters per workgroup
constexpr int kResStage = 2048;      // output staging bytes per compute wave

struct ResGeom {
    int TH, TW;          // output block
    int PH, PW;          // input patch
    int PWp;             // PW rounded up to a multiple of 16: pixels per patch row in LDS
    int tiles_h, tiles_w;
    int total_tiles;
    int tiles_base, tiles_rem;   // workgroup i owns tiles_base (+1 if i < tiles_rem) consecutive blocks
    int KS;              // channel slices of 32
    int NR;              // patch regions in LDS (2 .. 4); phase p uses region p % NR
    int slice_bytes;     // LDS bytes of one patch region (multiple of 1024)
    int w_bytes;         // LDS bytes of the filters: R*S*C*128
    int patch_loads;     // wave-wide loads per patch slice: PH * PWp / 16
    int skew;            // 1: odd patch rows store their chunks with bit 1 of the chunk number flipped (see the kernel)
    float inv_tw;
};

struct ResTile {
    int n, p0, q0;
};

__device__ __forceinline__ ResTile res_decode(int t, const ResGeom& g) {
    ResTile c;
    const int tile_w = t % g.tiles_w; t /= g.tiles_w;
    const int tile_h = t % g.tiles_h;
    c.n = t / g.tiles_h;
    c.p0 = tile_h * g.TH; c.q0 = tile_w * g.TW;
    return c;
}

// s_waitcnt vmcnt(n) for a wave-uniform run-time n (n >= 63 waits for nothing more than vmcnt(63))
__device__ __forceinline__ void wait_vmcnt_dyn(int n) {
    switch (n) {
#define ICONV_W(k) case k: wait_vmcnt<k>(); break;
        ICONV_W(0) ICONV_W(1) ICONV_W(2) ICONV_W(3) ICONV_W(4) ICONV_W(5) ICONV_W(6) ICONV_W(7)
        ICONV_W(8) ICONV_W(9) ICONV_W(10) ICONV_W(11) ICONV_W(12) ICONV_W(13) ICONV_W(14) ICONV_W(15)
        ICONV_W(16) ICONV_W(17) ICONV_W(18) ICONV_W(19) ICONV_W(20) ICONV_W(21) ICONV_W(22) ICONV_W(23)
        ICONV_W(24) ICONV_W(25) ICONV_W(26) ICONV_W(27) ICONV_W(28) ICONV_W(29) ICONV_W(30) ICONV_W(31)
        ICONV_W(32) ICONV_W(33) ICONV_W(34) ICONV_W(35) ICONV_W(36) ICONV_W(37) ICONV_W(38) ICONV_W(39)
        ICONV_W(40) ICONV_W(41) ICONV_W(42) ICONV_W(43) ICONV_W(44) ICONV_W(45) ICONV_W(46) ICONV_W(47)
#undef ICONV_W
        default: wait_vmcnt<0>(); break;
    }
}

template <typename T, typename TO, int MF, int S_>
__global__ void __launch_bounds__((kResWaves + kResLoaders) * 64)
ires_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const ResGeom g) {
    typedef typename Elem<T>::frag frag_t;
    constexpr int NWAVES = kResWaves + kResLoaders;
    // [filters: (slice, tap, filter 0..63) x 64 B][NR patch regions: padded patch pixel x 64 B][staging: 2 KiB per compute wave]
    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int t_begin = wg * g.tiles_base + min(wg, g.tiles_rem);
    const int t_end = t_begin + g.tiles_base + (wg < g.tiles_rem ? 1 : 0);
    const int RS = s.R * S_;
    const int phases = (t_end - t_begin) * g.KS;             // (block, channel slice) pairs of this workgroup
    if (phases <= 0) return;

    // ---- global -> LDS loads of one phase, split over `nparts` waves (this wave is `part`).
    // A wave-wide load fills 16 rows of 64 bytes: lane l fetches row l/4 of the group and the
    // logical chunk that lives at physical chunk l%4 of that row.  Patch rows are padded to a
    // multiple of 16 pixels and the filters of a tap come in groups of 16, so the row number
    // within the group alone decides the swizzle: the lane's chunk is the same for every load.
    const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * s.C * 2u;
    const uint32_t w_bytes = (uint32_t)s.K * s.Kg * 2u;
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
    const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds;
    const int l_row = lane >> 2;
    const int l_chunk = (lane & 3) ^ ((l_row >> 2) & 3);
    const uint32_t x_lane = (uint32_t)(l_row * s.C + l_chunk * 8) * 2u;       // byte offset of the lane within a 16-pixel group
    const uint32_t w_lane = (uint32_t)(l_row * s.Kg + l_chunk * 8) * 2u;      // ... within a 16-filter group
    const int groups = g.PWp >> 4;                                            // 16-pixel groups per patch row
    // Returns the number of loads this wave issued (the same for every lane).
    auto issue_loads = [&](int phase, int part, int nparts) {
        const int ks = phase % g.KS;
        int issued = 0;
        if (phase < g.KS) {
            // filters of this slice (first block only): load j covers tap j/4, filters 16*(j%4) + l/4
            for (int j = part; j < RS * 4; j += nparts, ++issued) {
                const int f0 = (j & 3) * 16;
                const uint32_t off = (uint32_t)(f0 * s.Kg + (j >> 2) * s.C + ks * 32) * 2u + w_lane;
                dma16(w_rsrc, f0 + l_row < s.K ? off : w_bytes,
                      (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + (uint32_t)((ks * RS * 4 + j) * 1024))));
            }
        }
        const ResTile tc = res_decode(t_begin + phase / g.KS, g);
        const int h_org = tc.p0 * s.stride - s.pad, w_org = tc.q0 * s.stride - s.pad;
        const uint32_t region = lds_base + (uint32_t)g.w_bytes + (uint32_t)(phase % g.NR) * (uint32_t)g.slice_bytes;
        int row = part / groups, grp = part - row * groups;             // load j = row * groups + grp
        const int drow = nparts / groups, dgrp = nparts - drow * groups;
        for (int j = part; j < g.patch_loads; j += nparts, ++issued) {
            const int h = h_org + row, w0 = w_org + grp * 16;
            const bool row_ok = (unsigned)h < (unsigned)s.H;                // uniform
            const uint32_t base = (uint32_t)(((tc.n * s.H + h) * s.W + w0) * s.C + ks * 32) * 2u;   // uniform; wraps when out of range
            const bool ok = row_ok & ((unsigned)(w0 + l_row) < (unsigned)s.W);
            const uint32_t flip = (uint32_t)(g.skew & row & 1) << 5;       // odd patch rows: chunk bit 1 flipped (32 bytes)
            dma16(x_rsrc, ok ? base + (x_lane ^ flip) : x_bytes, (uint32_t)__builtin_amdgcn_readfirstlane((int)(region + (uint32_t)(j * 1024))));
            grp += dgrp; row += drow;
            if (grp >= groups) { grp -= groups; ++row; }
        }
        return issued;
    };

    issue_loads(0, wave, NWAVES);               // the first phase's loads are shared by all waves

    if (wave >= kResWaves) {
        // =========================== loader waves ===========================================
        // Phase q may be loaded once phase q - NR (the previous user of its region) has been
        // computed by every wave, i.e. after barrier q - NR + 1.  The host keeps a wave's loads of
        // NR - 1 phases plus its share of the first phase below the 6-bit range of vmcnt.
        __builtin_amdgcn_s_setprio(3);          // few instructions, on the critical path: ahead of the compute waves at the arbiter
        const int lw = wave - kResWaves;
        // W: the phase the next wait is for.  later_i: loads this wave has issued for phase W + 1 + i
        // (NR <= 4, so at most W + 2 is in flight at a wait); after = their sum.
        int later0 = 0, later1 = 0, after = 0, issued_upto = 0;
        for (int p = 0; p < phases; ++p) {
            wait_vmcnt_dyn(after);              // W = p: everything up to phase p has landed
            __syncthreads();                    // phase p is in LDS; every wave has finished phase p - 1
            after -= later0;                    // W = p + 1
            later0 = later1; later1 = 0;
            while (issued_upto + 1 < phases && issued_upto + 1 <= p + g.NR - 1) {
                const int q = ++issued_upto;
                const int c = issue_loads(q, lw, kResLoaders);
                const int i = q - (p + 2);      // q = (W + 1) + i; i < 0: q is the phase waited for next
                if (i == 0) { later0 = c; after += c; }
                if (i == 1) { later1 = c; after += c; }
            }
        }
        return;
    }

    // =============================== compute waves ==============================================
    const int frow = lane & 31, fk = lane >> 5;
    const int m_half = wave >> 1, nh = wave & 1;
    const int npx = g.TH * g.TW;
    const char* lds_b = reinterpret_cast<const char*>(lds);
    // Byte offset in a patch region of the lane's operand of fragment mf, tap column s, filter row 0
    // and K step 0: pixel (th*stride, tw*stride + s*dil) of the padded patch, chunk l/32 (K step 1:
    // chunk 2 + l/32, i.e. the offset xor 32).  A filter row further down adds a multiple of 1 KiB,
    // which leaves the swizzle bits alone, so one add per operand read is all the arithmetic.
    uint32_t a_addr[MF][S_];
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) {
        const int t = (m_half * MF + mf) * 32 + frow;
        const int th = (int)(((float)t + 0.5f) * g.inv_tw);
        const int tw = t - th * g.TW;
#pragma unroll
        for (int sc = 0; sc < S_; ++sc) {
            const int pix = t < npx ? (th * g.PWp + tw) * s.stride + sc * s.dil : sc * s.dil;
            const int odd_row = t < npx ? (g.skew & th & 1) << 1 : 0;           // skew implies stride 1: patch row = th
            a_addr[mf][sc] = (uint32_t)(pix * 64 + ((fk ^ ((pix >> 2) & 3) ^ odd_row) << 4));
        }
    }
    const uint32_t row_step = (uint32_t)(s.dil * g.PWp * 64);
    // filter fragment of (slice, tap, K step kk): filter f = 32*nh + l%32, chunk 2*kk + l/32
    const int f_lane = nh * 32 + frow;
    const uint32_t b_lane0 = (uint32_t)(f_lane * 64 + ((fk ^ ((f_lane >> 2) & 3)) << 4));
    const uint32_t b_lane1 = b_lane0 ^ 32u;
    // output staging, 16 pixels x 32 filters at a time: piece c (16 bytes, 4 filters) of pixel i at
    // stage_off(i, c)
    char* stg = reinterpret_cast<char*>(lds) + g.w_bytes + g.NR * g.slice_bytes + wave * kResStage;
    const int f16 = frow & 15;
    const uint32_t sw0 = stage_off(f16, fk);        // piece 2*gq + fk: xor (gq << 5)
    const int l8 = lane >> 3, c8 = lane & 7;
    const uint32_t sr0 = stage_off(l8, c8);          // pixel l/8 (+8), piece l%8
    const uint32_t sr1 = stage_off(l8 + 8, c8);
    const size_t y_elems = (size_t)s.M * s.K;
    const bool k_ok = nh * 32 + 4 * c8 + 3 < s.K;

    wait_vmcnt<0>();                            // this wave's share of the first phase's loads
    floatx16 acc[MF];

    // ---- the K loop of phase p (one channel slice of a block) for fragments MF0 .. MF1-1.
    // K steps of a filter row r: (s, kk) = (0,0), (0,1), (1,0), ... (S-1, 1); kk selects 16 of the
    // slice's 32 channels.  In every step the filter fragment of the next step is read into the
    // other B register set first, and each pixel fragment is re-read for the next step as soon as
    // its MFMA has been issued, so the LDS reads of a step run under the MFMAs of the step before.
    // (After the last row the reads repeat it: unconditional, and harmless.)  The scheduling
    // barriers keep that order.
    auto compute_slice = [&](int p, auto mf0_t, auto mf1_t) {
        constexpr int MF0 = decltype(mf0_t)::value, MF1 = decltype(mf1_t)::value;
        const int ks = p % g.KS;
        const uint32_t pa = lds_base + (uint32_t)(g.w_bytes + (p % g.NR) * g.slice_bytes);   // LDS address of the patch region
        const char* pb = lds_b + ks * RS * 4096;
        frag_t af[MF], b0, b1;
        // (one instruction, (a ^ mask) + row offset, written out so that the optimiser neither splits it
        // nor keeps the xor-ed variants of all addresses in registers across the loop; mask is 0 or 32 in a
        // scalar register -- K step and row skew -- and the row offset travels in a vector register,
        // because a VOP3 instruction reads one scalar operand at most)
        auto fetch_a = [&](int mf, int sc, uint32_t mask, uint32_t roff_v) {
            uint32_t addr;
            asm volatile("v_xad_u32 %0, %1, %2, %3" : "=v"(addr) : "v"(a_addr[mf][sc]), "s"(mask), "v"(roff_v));
            return *reinterpret_cast<const frag_t __attribute__((address_space(3)))*>(addr);
        };
        auto fetch_b = [&](int tap, int kk) {
            return *reinterpret_cast<const frag_t*>(pb + tap * 4096 + (kk ? b_lane1 : b_lane0));
        };
        // flipped(r): the patch rows filter row r reads have chunk bit 1 flipped relative to filter row 0
        // (skewed layout, odd r*dil), which swaps the roles of the two K steps in the address arithmetic.
        auto flipped = [&](int r) { return (uint32_t)(g.skew & (min(r, s.R - 1) * s.dil) & 1) << 5; };
        auto row = [&](int r, auto first) {
            const int r_next = min(r + 1, s.R - 1);
            uint32_t roff = pa + (uint32_t)r * row_step, roff_next = pa + (uint32_t)r_next * row_step;
            asm volatile("" : "+v"(roff), "+v"(roff_next));       // one copy each in vector registers for the whole row
            const uint32_t mask_c = flipped(r), mask_n = flipped(r + 1);
#pragma unroll
            for (int st = 0; st < 2 * S_; ++st) {
                const bool wrap = st + 1 == 2 * S_;                   // next step: first of the next row
                const int sc_n = wrap ? 0 : (st + 1) >> 1, kk_n = wrap ? 0 : (st + 1) & 1;
                frag_t& bc = (st & 1) ? b1 : b0;
                frag_t& bn = (st & 1) ? b0 : b1;
                bn = fetch_b((wrap ? r_next : r) * S_ + sc_n, kk_n);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int mf = MF0; mf < MF1; ++mf) {
                    if (decltype(first)::value && st == 0) {
                        floatx16 z;
#pragma unroll
                        for (int v = 0; v < 16; ++v) z[v] = 0.f;
                        acc[mf] = Elem<T>::mfma32(bc, af[mf], z);
                    } else {
                        acc[mf] = Elem<T>::mfma32(bc, af[mf], acc[mf]);
                    }
                    af[mf] = fetch_a(mf, sc_n, (wrap ? mask_n : mask_c) ^ (uint32_t)(kk_n << 5), wrap ? roff_next : roff);
                    __builtin_amdgcn_sched_barrier(0);
                }
            }
        };
        b0 = fetch_b(0, 0);
#pragma unroll
        for (int mf = MF0; mf < MF1; ++mf) af[mf] = fetch_a(mf, 0, 0u, pa);
        __builtin_amdgcn_sched_barrier(0);
        if (ks == 0) row(0, std::true_type{});  // a block's first step starts the accumulators
        else row(0, std::false_type{});
        for (int r = 1; r < s.R; ++r) row(r, std::false_type{});
    };

    // ---- the epilogue of a block for fragments MF0 .. MF1-1.  The filters are the MFMA's row
    // operand: lane l holds pixel l%32 of fragment mf and, in accumulator element v, filter
    // 32*nh + 8*(v/4) + 4*(l/32) + v%4.  Half a fragment (16 pixels x 32 filters) at a time goes
    // through the wave's staging area (in-order LDS, no wait needed in between) and leaves as
    // 16-byte pieces, 8 lanes per pixel = one 128-byte line of the y row.
    auto epilogue = [&](int tile, auto mf0_t, auto mf1_t) {
        constexpr int MF0 = decltype(mf0_t)::value, MF1 = decltype(mf1_t)::value;
        const ResTile tc = res_decode(tile, g);
        const size_t org = ((size_t)(tc.n * s.P + tc.p0) * s.Q + tc.q0) * s.K;
        const size_t rem = (y_elems - org) * sizeof(TO);
        const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + org, 0, rem > 0xffffffffull ? 0xffffffffu : (uint32_t)rem,
                                                               kRsrcFlags);
        // (opaque to the optimiser: the pixel arithmetic below is then redone per block instead of
        // being kept in registers across the K loop, which has none to spare)
        int l8v = l8;
        asm volatile("" : "+v"(l8v));
#pragma unroll
        for (int mf = MF0; mf < MF1; ++mf) {
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
                    const int t = (m_half * MF + mf) * 32 + h * 16 + 8 * j + l8v;
                    const int th = (int)(((float)t + 0.5f) * g.inv_tw);
                    const int tw = t - th * g.TW;
                    const bool ok = k_ok & (t < npx) & (tc.p0 + th < s.P) & (tc.q0 + tw < s.Q);
                    const uint32_t off = (uint32_t)((th * s.Q + tw) * s.K + nh * 32 + 4 * c8) * (uint32_t)sizeof(TO);
                    if (ok) store_piece<TO>(out[h][j], y_rsrc, off);
                }
        }
    };

    // (Computing and storing a single block in two groups of fragments, so that the first group's
    // stores drain under the second group's MFMAs, was measured and is slower: a wave's stores
    // block it for as long as the memory system takes to accept them.)
    constexpr std::integral_constant<int, 0> kZero{};
    constexpr std::integral_constant<int, MF> kAll{};
    for (int p = 0; p < phases; ++p) {
        __syncthreads();                        // phase p is in LDS
        compute_slice(p, kZero, kAll);
        if (p % g.KS + 1 == g.KS) epilogue(t_begin + p / g.KS, kZero, kAll);
    }
}

constexpr int kResLdsLimit = 160 * 1024;

// Chooses the output block TH x TW (TH*TW <= 64*MF) for a fragment count MF.  Cost model as for
// the patch-reuse kernels: MFMA work of all (padded) blocks plus the patch pixels brought into LDS.
bool plan_res(const ConvShape& s, int MF, ResGeom* g, double* cost_out) {
    if ((s.C % 32) != 0 || (s.K & 3) != 0 || s.K > kResBN) return false;
    if (s.S != 1 && s.S != 3) return false;                    // the filter width is a compile-time parameter
    if (MF == 8 && s.S == 3) return false;                     // eight fragments and three address sets exceed the register file
    const int BM = 2 * MF * 32;          // two pixel halves of MF fragments; the wave pairs split the filters
    const int RS = s.R * s.S;
    const long w_lds = (long)s.Kg * 128;
    const int KS = s.C / 32;
    double best = 1e300;
    bool found = false;
    for (int tw = 1; tw <= s.Q && tw <= BM; ++tw) {
        int th = BM / tw;
        if (th > s.P) th = s.P;
        if (th < 1) continue;
        const int ph = (th - 1) * s.stride + (s.R - 1) * s.dil + 1;
        const int pw = (tw - 1) * s.stride + (s.S - 1) * s.dil + 1;
        const int pwp = (pw + 15) & ~15;
        const long patch_loads = (long)ph * (pwp / 16);
        const long slice_bytes = patch_loads * 1024;
        // patch regions: one per channel slice when that fits (at most three), else two
        int NR = KS < 2 ? 2 : (KS > 3 ? 3 : KS);
        while (NR > 2 && w_lds + NR * slice_bytes + kResWaves * kResStage > kResLdsLimit) --NR;
        if (w_lds + NR * slice_bytes + kResWaves * kResStage > kResLdsLimit) continue;
        if ((long)ph * pwp >= (1 << 20)) continue;
        // a loader wave's loads of NR - 1 phases (patch and, in the first block, filters) and its
        // share of the first phase must stay countable by vmcnt
        const long per_phase = (patch_loads + kResLoaders - 1) / kResLoaders + (RS * 4 + kResLoaders - 1) / kResLoaders;
        if ((NR - 1) * per_phase + per_phase / 2 + 2 > 47) continue;
        if ((long)th * s.Q * s.K * 4 >= (1L << 31)) continue;             // in-block output offsets are 32-bit
        const long tiles = (long)((s.P + th - 1) / th) * ((s.Q + tw - 1) / tw);
        const double cost = (double)tiles * ((double)BM * RS + 4.0 * (double)ph * pwp);
        if (cost < best) {
            best = cost;
            found = true;
            g->TH = th; g->TW = tw; g->PH = ph; g->PW = pw; g->PWp = pwp;
            g->tiles_h = (s.P + th - 1) / th; g->tiles_w = (s.Q + tw - 1) / tw;
            g->KS = KS; g->NR = NR; g->slice_bytes = (int)slice_bytes; g->w_bytes = (int)w_lds;
            g->patch_loads = (int)patch_loads;
            g->inv_tw = 1.0f / (float)tw;
            g->skew = (s.stride == 1 && (tw & 15) == 8) ? 1 : 0;
        }
    }
    if (!found) return false;
    const long total = (long)s.N * g->tiles_h * g->tiles_w;
    if (total > 0x7fffffffL || RS * 4 * 1024L * KS != w_lds) return false;
    g->total_tiles = (int)total;
    if (cost_out) *cost_out = best * (double)s.N;
    return true;
}

template <typename T, typename TO, int MF, int S_>
hipError_t launch_res_t(const void* x, const void* w, void* y, const ConvShape& s, ResGeom g, hipStream_t st) {
    const int lds_bytes = g.w_bytes + g.NR * g.slice_bytes + kResWaves * kResStage;
    auto kern = ires_kernel<T, TO, MF, S_>;
    const int threads = (kResWaves + kResLoaders) * 64;
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kResLdsLimit);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    static std::atomic<long long> occ_slot{-1};
    const int occ = cached_occupancy(occ_slot, (const void*)kern, threads, lds_bytes);
    const int cap = call_max_workgroups();
    const long slots = cap > 0 ? cap : (long)device_cus() * occ;
    const long per = (g.total_tiles + slots - 1) / slots;
    const int nwg = (int)((g.total_tiles + per - 1) / per);
    g.tiles_base = g.total_tiles / nwg;
    g.tiles_rem = g.total_tiles % nwg;
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(threads), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y, s, g);
    return hipGetLastError();
}

template <int MF, int S_>
hipError_t launch_res_ms(const void* x, const void* w, void* y, const ConvShape& s, const ResGeom& g, int in_t, int out_t,
                         hipStream_t st) {
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_res_t<bf16_t, float, MF, S_>(x, w, y, s, g, st);
        return launch_res_t<bf16_t, bf16_t, MF, S_>(x, w, y, s, g, st);
    }
    if (out_t == OUT_F32) return launch_res_t<f16_t, float, MF, S_>(x, w, y, s, g, st);
    return launch_res_t<f16_t, f16_t, MF, S_>(x, w, y, s, g, st);
}

template <int MF>
hipError_t launch_res_mf(const void* x, const void* w, void* y, const ConvShape& s, const ResGeom& g, int in_t, int out_t,
                         hipStream_t st) {
    if (s.S == 1) return launch_res_ms<MF, 1>(x, w, y, s, g, in_t, out_t, st);
    return launch_res_ms<MF, 3>(x, w, y, s, g, in_t, out_t, st);
}

constexpr int kResMF[] = {7, 8};
// r: channel-slice phases (this file); t: filter-row phases, whole pixels per LDS row (iconv_rowres.hip)
const char* const kResNames[] = {"r448x64_f7_4+4", "r512x64_f8_4+4", "t448x64_f7_4+4", "t512x64_f8_4+4", "s448x64_f7_8", "s512x64_f8_8"};
constexpr int kNumRes = 6;

}  // namespace

int resident_num_variants() { return kNumRes; }
const char* resident_variant_name(int v) { return kResNames[v]; }

bool resident_supported(const ConvShape& s, int v) {
    if (v >= 2) return rowres_supported(s, v - 2);
    ResGeom g;
    return v >= 0 && plan_res(s, kResMF[v], &g, nullptr);
}

// The variant with the lower modelled cost, or -1 when the layer does not fit the kernels.
// Their blocks are large (448 or 512 pixels x all filters), so they are only offered when there are
// enough of them to occupy most of the device -- or half of it, when the 256-pixel tiles of the
// patch-reuse kernel that would run instead no longer fit one round of workgroups (measured on the
// 56 x 56, 64 -> 64 layer: batches 20 .. 27 take 13.2 .. 14.3 us here against 16.6 us there).
// Layers with 32 or 64 channels take the filter-row-phased kernel, which starts its first MFMA sooner.
int resident_choose(const ConvShape& s) {
    const long cus = device_cus();
    // full-width tiles of 256 / Q output rows, as the patch-reuse planner forms them for narrow maps
    const long th = s.Q <= 256 ? 256 / s.Q : 1;
    const long patch_tiles = (long)s.N * ((s.P + th - 1) / th) * ((s.Q + 255) / 256);
    const long enough = patch_tiles > cus ? cus / 2 : cus * 3 / 4;
    int best = -1;
    double best_cost = 0;
    for (int v = 0; v < kNumRes; ++v) {
        double c = 0;
        long blocks = 0;
        bool ok;
        if (v >= 2) {
            ok = rowres_plan_cost(s, v - 2, &c, &blocks);
        } else {
            ResGeom g;
            ok = plan_res(s, kResMF[v], &g, &c);
            blocks = ok ? g.total_tiles : 0;
        }
        if (!ok || blocks < enough) continue;
        // the all-compute form ("s") has one block per workgroup: it is for launches of one round of workgroups,
        // where it measured 6-16 % faster; with more blocks the persistent forms load the next block under the stores
        if (v >= 4 && blocks > cus) continue;
        // on equal cost: filter-row phases ("t") before channel-slice phases ("r"), all-compute ("s") before both
        if (best < 0 || c < best_cost || (c <= best_cost && ((v >= 2 && best < 2) || (v >= 4 && best < 4)))) {
            best = v;
            best_cost = c;
        }
    }
    return best;
}

hipError_t launch_resident(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v,
                           hipStream_t st) {
    if (v >= 2) return launch_rowres(x, w, y, s, in_t, out_t, v - 2, st);
    ResGeom g;
    if (v < 0 || !plan_res(s, kResMF[v], &g, nullptr)) return hipErrorInvalidConfiguration;
    if (v == 0) return launch_res_mf<7>(x, w, y, s, g, in_t, out_t, st);
    return launch_res_mf<8>(x, w, y, s, g, in_t, out_t, st);
}

}  // namespace iconv

// Implicit channel-first im2col with inter-tile reuse (paper section 5, "Inter-tile Reuse").
//
// The lowered-matrix sub-tiles of neighbouring filter taps overlap almost completely, and the
// paper reorders the K loop so that consecutive sub-tiles reuse on-chip data.  This kernel takes
// that to its end: the K loop runs channel chunk OUTER, tap (r, s) INNER, and for one channel
// chunk the input footprint of the whole output tile (a TH x TW block of output pixels of one
// image, i.e. a PH x PW patch of input pixels, zero where it leaves the image) is placed in LDS
// once.  All R*S taps then read their A operands from that patch: the A row of output pixel
// (th, tw) for tap (r, s) is patch pixel (th*stride + r*dil, tw*stride + s*dil), a channel-
// contiguous run exactly as in section 3.1.  Global -> LDS traffic for the input drops by about
// R*S / ((PH*PW)/(TH*TW)); the filter tile of each step still streams through a small ring.
//
// Tiling follows section 5's block-level scheme: one workgroup per (image, output block,
// BN filters), no atomics.  A feature map that fits a tile at least twice is stacked: the tile
// then holds several whole images, their patches one below the other in LDS, so that the small
// maps at the end of a network fill the rows of the MFMA tiles.
#include <algorithm>
#include <atomic>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

struct PatchGeom {
    int TH, TW;          // output block
    int PH, PW;          // input patch
    int npix;            // PH*PW
    int tiles_h, tiles_w, tiles_n;
    int a_blocks;        // wave-wide patch loads per wave and channel chunk
    int dph, dpw;        // (WAVES*RPB) / PW and % PW: patch-pixel step between a lane's loads
    int patch_bytes;     // LDS bytes of one patch buffer (multiple of 1024)
    int total_tiles;     // N * tiles_h * tiles_w * tiles_n
    int tiles_per_wg;    // contiguous tiles per workgroup
    float inv_tw;        // 1 / TW
    // Small feature maps: a tile holds G whole images (TH = P, TW = Q), stacked along the rows: output
    // row v of the tile is row v % TH of image v / TH, patch row v is row v % PH of image v / PH.
    int G;               // images per tile (1 unless the whole map fits a tile at least twice)
    float inv_th, inv_ph;
    // Tile order.  0: filter tile fastest (neighbouring workgroups share an input patch).  1: filter tile slowest, so
    // that the workgroups of one XCD (a contiguous range of tile numbers) read few filter tiles and these stay in that
    // XCD's L2 -- for layers whose filters outweigh their input (the 7 x 7 maps with 512 channels).
    int n_slow;
    int tiles_m;         // tiles per filter tile (total_tiles / tiles_n)
};

// Patch swizzle.  The patch is an array of 256-byte windows (all 64 LDS banks), each holding
// PPW = 16/CPR pixels of CPR 16-byte chunks.  Chunk c of pixel pp has logical slot
// (pp % PPW)*CPR + c in window pp / PPW and lives at physical slot  logical ^ (window & 15) for even strides,
// (window & (CPR-1)) for odd strides: an MFMA operand read has its 16 consecutive lanes on 16
// pixels that are `stride` apart, same chunk.  For an odd stride those pixels spread evenly over
// the pixel-in-window positions, and XOR-ing the window number into the chunk bits alone makes
// the 16 slots distinct; for an even stride they share few pixel-in-window positions, and the
// window number has to be XOR-ed into all four slot bits.  (Where the 32 pixels of a fragment run
// from one block row into the next, their patch pixels jump by PW - TW and two lane groups of a
// pass can meet in a slot.  Taking the XOR term from the block-linear pixel index instead removes
// those conflicts, was measured, and is 1-3 % SLOWER on the 64 x 64 dilated and the 7 x 7 layers:
// the two extra integer operations per fragment and step, and per load in the loader waves, cost
// more than the conflicts, which these loops hide under their MFMAs.)
//
// Wave roles.  The workgroup has WAVES_M*WAVES_N compute waves and NLD loader waves.  Loader waves
// only issue the global -> LDS loads (their address arithmetic then overlaps the compute waves'
// MFMAs instead of delaying them); compute waves only read LDS, issue MFMAs and store results.
// All waves meet at one barrier per K step.
//
// Persistence.  A workgroup owns a contiguous range of output tiles and walks through them as
// one sequence of phases (tile, channel chunk).  While a phase is computed the loader waves
// bring in the patch of the next phase -- the next chunk of the same tile or the first chunk of
// the next tile -- into the other patch buffer, and the filter ring simply runs on across tile
// boundaries.
//
// Output.  With SS == 0 the compute waves store their accumulators themselves.  That stalls
// them for as long as the memory system takes to accept a tile (the write of y is the largest
// traffic of the low-channel layers), so with SS > 0 they only drop the finished tile into an
// LDS staging buffer (fp32, 16-byte pieces, XOR-swizzled by pixel) and go on with the next tile,
// while NSW store waves drain the staging buffer to y -- SS wave-wide 16-byte-per-lane stores
// per K step, whole row pieces per 16 lanes -- during the steps of the next tile.  The drain of
// a tile ends one step before that tile's last, so the barrier of the last step separates it
// from the compute waves' next deposit; the last tile is drained after one extra barrier at the
// end.  Store waves are separate from loader waves because a wave that counts outstanding loads
// with s_waitcnt vmcnt must not have stores in flight as well: stores need not retire in order
// with loads.  The last tile of a workgroup, whose stores nothing can hide, leaves through
// wave-private LDS staging areas instead, so that every store covers whole 128-byte lines.
//
// Prefetching variants (PF).  A wave issues in order, so only what sits between two of its
// MFMAs runs in their shadow.  With PF the operand fragments of the next group of K slices, and
// the addresses of the next step, are requested between the MFMAs of the current group, across
// the step barrier too; the loaders then keep the NEXT step's filter tile complete at every
// barrier, and the fragment registers act as one more stage of the ring.
struct TileCoord {
    int n, p0, q0, k0;
};

template <int BN> __device__ __forceinline__ TileCoord decode_tile(int t, const PatchGeom& g) {
    TileCoord c;
    int tile_n;
    if (g.n_slow) {
        tile_n = t / g.tiles_m;
        t -= tile_n * g.tiles_m;
    } else {
        tile_n = t % g.tiles_n;
        t /= g.tiles_n;
    }
    const int tile_w = t % g.tiles_w; t /= g.tiles_w;
    const int tile_h = t % g.tiles_h;
    c.n = (t / g.tiles_h) * g.G;
    c.p0 = tile_h * g.TH; c.q0 = tile_w * g.TW; c.k0 = tile_n * BN;
    return c;
}

template <int V> struct IntTag { static constexpr int value = V; };

template <typename T, typename TO, int CB, int WAVES_M, int WAVES_N, int MI, int NI, int STB, int LA, int NLD, int SS, int NSW,
          int PF, int KS>
__global__ void __launch_bounds__((WAVES_M * WAVES_N * KS + NLD + NSW) * 64)
ipatch_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const PatchGeom g) {
    // KS == 2: two compute waves per tile position, each with the K slices of one half of every step (so that every
    // SIMD has two waves issuing MFMAs while a wave still owns a 32 x 64 output); their partial sums meet in LDS
    // after the last step.  Only for workgroups with one tile, whole 16-byte output pieces and no prefetch pipeline.
    constexpr int WAVES_P = WAVES_M * WAVES_N;  // tile positions
    constexpr int WAVES_C = WAVES_P * KS;       // compute waves
    static_assert(KS == 1 || (KS == 2 && PF == 0 && SS == 0 && CB >= 64), "K split: two halves of the plain loop");
    constexpr int CPR = CB / 8;                 // 16-byte chunks per pixel (or filter row) and channel chunk
    constexpr int RPB = 64 / CPR;               // pixels (filter rows) one wave-wide load covers
    constexpr int PPW = 16 / CPR;               // pixels per 256-byte LDS window
    constexpr int BN = WAVES_N * NI * 32;
    constexpr int B_IT = BN / RPB / NLD;        // filter-tile loads per loader wave per step
    constexpr int KI = CB / 16;
    constexpr int PIX_BYTES = CB * 2;
    constexpr int BSTAGE_BYTES = BN * PIX_BYTES;
    static_assert(BN % (RPB * NLD) == 0 && B_IT >= 1, "filter tile must divide over the loader waves");
    static_assert(NLD % 4 == 0, "the patch loader needs a multiple of four loader waves");
    constexpr int BM = WAVES_M * MI * 32;
    constexpr int SPR = BN / 4;                 // 16-byte fp32 pieces per staging row (one output pixel)
    constexpr int ST_ROWS = 64 / SPR;           // staging rows one wave-wide store covers
    constexpr int ST_IT = SS > 0 ? BM / ST_ROWS / (NSW > 0 ? NSW : 1) : 0;   // wave-wide stores per store wave per tile
    static_assert((STB - 2) * B_IT + (STB - 1) * LA < 64, "too many loads in flight for vmcnt");
    static_assert(PF == 0 || (STB >= 3 && SS == 0), "the prefetching pipeline needs three filter stages and stores its own output");
    // Steady-state loads that may stay in flight when a step's barrier is reached.  Without
    // prefetch the step's own filter tile must have landed; with prefetch (PF) the NEXT step's must.
    constexpr int WAIT_STEP = PF ? (STB - 3) * B_IT + (STB - 2) * LA : (STB - 2) * B_IT + (STB - 1) * LA;
    static_assert((SS == 0 && NSW == 0) || (SS > 0 && NSW > 0 && BM % (ST_ROWS * NSW) == 0 && SPR <= 64),
                  "staging rows must divide over the store waves");
    typedef typename Elem<T>::frag frag_t;

    // [patch 0][patch 1][STB filter stages][1 KiB sink per loader wave][staging BM x BN fp32 if SS > 0]
    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int t_begin = wg * g.tiles_per_wg;
    const int t_end = min(t_begin + g.tiles_per_wg, g.total_tiles);
    const int RS = s.R * s.S;
    const int chunks = (s.C + CB - 1) / CB;
    const int phases = (t_end - t_begin) * chunks;           // (tile, channel chunk) pairs of this workgroup
    const int steps = phases * RS;
    const uint32_t bstage_off = 2u * (uint32_t)g.patch_bytes;   // byte offset of the filter ring
    const uint32_t staging_off = bstage_off + STB * BSTAGE_BYTES + NLD * 1024;   // byte offset of the staging buffer
    const int steps_per_tile = chunks * RS;
    // which bits of the window number the patch swizzle XORs into the slot number (see above)
    const int wmask = (s.stride & 1) ? (CPR - 1) : 15;

    if (wave >= WAVES_C && wave < WAVES_C + NLD) {
        // =========================== loader waves ===========================================
        // Their instructions are few but on the critical path of every step: they take priority over
        // the compute waves (which spend their time in MFMAs) at the instruction arbiter.
        __builtin_amdgcn_s_setprio(3);
        const int lw = wave - WAVES_C;
        const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * s.C * 2u;
        const uint32_t w_bytes = (uint32_t)s.K * s.Kg * 2u;
        const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
        const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
        const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds;
        const uint32_t bstage_base = lds_base + bstage_off;
        const uint32_t sink = bstage_base + STB * BSTAGE_BYTES + lw * 1024;

        // ---- patch loads.  A wave-wide load fills four 256-byte windows; lane l owns physical slot
        // l%16 of window 4*jb + l/16 (jb = lw, lw + NLD, ...) and fetches the (pixel, chunk) whose
        // logical slot maps there.  Advancing jb by NLD (a multiple of four) leaves window & 15, and
        // so the lane's pixel-in-window and chunk, unchanged: the lane's pixel moves by NLD*RPB, and
        // its (row, column) in the patch is advanced incrementally.
        const int a_win0 = lw * 4 + (lane >> 4);
        const int a_slot = (lane & 15) ^ (a_win0 & wmask);
        const int a_lc = (a_slot % CPR) * 8;    // first channel (within a chunk) this lane fetches
        const int a_pp0 = a_win0 * PPW + a_slot / CPR;
        const int a_ph0 = a_pp0 / g.PW;
        const int a_pw0 = a_pp0 - a_ph0 * g.PW;
        int a_ph, a_pw, a_j;                    // running state within one phase
        // The lane's pixel as (image of the tile, row within that image's patch) and as a byte offset into x, all
        // advanced by additions: a load moves the pixel by dph rows and dpw columns (+ a row when the column wraps,
        // + an image when the row leaves the image's patch, which the host allows at most once per load).
        int a_gi = 0, a_phi = 0;
        uint32_t a_off = 0;
        // (modulo 2^32 throughout: an offset is only used when its pixel exists, and then it is below 2^31)
        const uint32_t a_step0 = (uint32_t)(g.dph * s.W + g.dpw) * (uint32_t)s.C * 2u;
        const uint32_t a_stepw = (uint32_t)(s.W - g.PW) * (uint32_t)s.C * 2u;
        const uint32_t a_stepg = (uint32_t)(s.H - g.PH) * (uint32_t)s.W * (uint32_t)s.C * 2u;
        int a_n = 0, a_hb = 0, a_wb = 0, a_c0 = 0, a_buf = 0;   // phase being loaded: image, patch origin, chunk, buffer
        bool a_live = false;
        auto patch_begin = [&](int phase) {     // point the patch loader at phase `phase` (or switch it off)
            a_ph = a_ph0; a_pw = a_pw0; a_j = 0;
            a_live = phase < phases;
            if (a_live) {
                const TileCoord tc = decode_tile<BN>(t_begin + phase / chunks, g);
                a_n = tc.n;
                a_hb = tc.p0 * s.stride - s.pad;
                a_wb = tc.q0 * s.stride - s.pad;
                a_c0 = (phase % chunks) * CB;
                a_buf = phase & 1;
                a_gi = g.G > 1 ? (int)(((float)a_ph + 0.5f) * g.inv_ph) : 0;
                a_phi = a_ph - a_gi * g.PH;
                a_off = (uint32_t)((((a_n + a_gi) * s.H + a_hb + a_phi) * s.W + a_wb + a_pw) * s.C + a_c0 + a_lc) * 2u;
            }
        };
        // one patch load (or a no-op load into the sink once the phase's patch is complete)
        auto patch_load = [&](bool allowed) {
            const int h = a_hb + a_phi, ww = a_wb + a_pw;
            const bool real = allowed && a_live && a_j < g.a_blocks;   // wave-uniform
            const bool ok = real & (a_ph < g.G * g.PH) & (a_n + a_gi < s.N) & ((unsigned)h < (unsigned)s.H) &
                            ((unsigned)ww < (unsigned)s.W) & ((a_c0 + a_lc) < s.C);
            const uint32_t dst = real ? lds_base + (uint32_t)a_buf * g.patch_bytes + (uint32_t)(lw + a_j * NLD) * 1024u : sink;
            dma16(x_rsrc, ok ? a_off : x_bytes, (uint32_t)__builtin_amdgcn_readfirstlane((int)dst));
            a_pw += g.dpw;
            const int wrap = a_pw >= g.PW ? 1 : 0;
            a_pw -= wrap ? g.PW : 0;
            a_ph += g.dph + wrap;
            a_phi += g.dph + wrap;
            a_off += a_step0 + (wrap ? a_stepw : 0u);
            if (g.G > 1) {                      // uniform
                const int cross = a_phi >= g.PH ? 1 : 0;
                a_phi -= cross ? g.PH : 0;
                a_gi += cross;
                a_off += cross ? a_stepg : 0u;
            }
            ++a_j;
        };

        // ---- filter-tile loads (one BN x CB tile per step)
        const int pc = lane % CPR, lr = lane / CPR;
        const bool ragged_c = (s.C % CB) != 0;
        // Offset of the lane's 16 bytes at tap (0, 0), chunk 0; filters past K carry w_bytes instead,
        // which stays out of range (a zero load) whatever tap offset is added: the host checks that
        // 2 * w_bytes fits 32 bits.
        uint32_t b_off[B_IT];
        int b_tile = t_begin;                   // tile whose filters the next load belongs to
        auto filter_tile = [&]() {
            const TileCoord tc = decode_tile<BN>(b_tile, g);
#pragma unroll
            for (int j = 0; j < B_IT; ++j) {
                const int row = (lw + j * NLD) * RPB + lr;
                b_off[j] = (tc.k0 + row) < s.K ? (uint32_t)((tc.k0 + row) * s.Kg + swz<CPR>(row, pc) * 8) * 2u : w_bytes;
            }
        };
        filter_tile();
        int lr_ = 0, ls_ = 0, lc0 = 0;          // tap (lr_, ls_) of channel chunk lc0 to load next
        auto filter_load = [&](int stage, bool live) {
            const uint32_t delta = (uint32_t)((lr_ * s.S + ls_) * s.C + lc0) * 2u;     // tap and chunk: uniform
            if (!live) {
                // a step past the end loads nothing (zeros), but keeps the count of loads in flight
#pragma unroll
                for (int j = 0; j < B_IT; ++j)
                    dma16(w_rsrc, w_bytes, bstage_base + (uint32_t)(stage * BSTAGE_BYTES + (lw + j * NLD) * 1024));
            } else if (ragged_c) {
#pragma unroll
                for (int j = 0; j < B_IT; ++j) {
                    const int row = (lw + j * NLD) * RPB + lr;
                    const bool ok = (lc0 + swz<CPR>(row, pc) * 8) < s.C;
                    dma16(w_rsrc, ok ? b_off[j] + delta : w_bytes,
                          bstage_base + (uint32_t)(stage * BSTAGE_BYTES + (lw + j * NLD) * 1024));
                }
            } else {
                // the common case costs no vector instruction but the load itself
#pragma unroll
                for (int j = 0; j < B_IT; ++j)
                    dma16s(w_rsrc, b_off[j], (uint32_t)__builtin_amdgcn_readfirstlane((int)delta),
                           bstage_base + (uint32_t)(stage * BSTAGE_BYTES + (lw + j * NLD) * 1024));
            }
            if (++ls_ == s.S) {
                ls_ = 0;
                if (++lr_ == s.R) {
                    lr_ = 0;
                    lc0 += CB;
                    if (lc0 >= s.C) {           // next tile
                        lc0 = 0;
                        if (++b_tile < t_end) filter_tile();
                    }
                }
            }
        };

        // prologue: the whole patch of phase 0, then what the STB-1 steps before the first one would
        // have issued (their filter tiles; no-op loads in place of patch slices), so that the
        // steady-state wait count holds from the first step on.  Loads complete in issue order, so
        // the first step's wait for its filter tile also covers the patch.
        patch_begin(0);
        for (int j = 0; j < g.a_blocks; ++j) patch_load(true);
#pragma unroll
        for (int j = 0; j < STB - 1; ++j) {
            filter_load(j, j < steps);
#pragma unroll
            for (int l = 0; l < LA; ++l) dma16(x_rsrc, x_bytes, sink);
        }
        if (PF) {
            // the compute waves read the first step's operands before the loop: stage 0 and patch 0
            wait_vmcnt<(STB - 2) * B_IT + (STB - 1) * LA>();
            __syncthreads();
        }
        int fill = STB - 1, step = 0;
        for (int phase = 0; phase < phases; ++phase) {
            patch_begin(phase + 1);
            for (int t = 0; t < RS; ++t, ++step) {
                // Everything issued after the filter tile that has to be complete may stay in flight
                // (without prefetch: STB-2 later filter tiles and STB-1 groups of patch loads).
                wait_vmcnt<WAIT_STEP>();
                __syncthreads();
                // The stage refilled here was read for the last time before the barrier just passed:
                // in step - 1, with prefetch partly in step - 2.
                filter_load(fill, step + STB - 1 < steps);
                // The next phase's patch arrives LA loads per step; the last STB-1 steps of a phase
                // carry no-op loads only, so the patch is complete once the next phase's first step
                // has waited (with prefetch: once the phase's last step has, which reads ahead).
#pragma unroll
                for (int l = 0; l < LA; ++l) patch_load(t <= RS - STB);
                fill = fill + 1 == STB ? 0 : fill + 1;
            }
        }
        wait_vmcnt<0>();
        if (SS > 0) __syncthreads();            // the barrier that hands the last tile to the store waves
        return;
    }

    if (SS > 0 && wave >= WAVES_C + NLD) {
        // =========================== store waves ============================================
        const int sw = wave - WAVES_C - NLD;
        // Store number j of a tile (j = 0 .. ST_IT-1) covers staging rows (sw + j*NSW)*ST_ROWS .. +ST_ROWS,
        // lane l: row +l/SPR, 16-byte piece l%SPR.
        const uint32_t y_bytes = (uint32_t)s.M * (uint32_t)s.K * (uint32_t)sizeof(TO);   // < 2^32 checked by the host
        const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y, 0, y_bytes, kRsrcFlags);
        const int npx = g.TH * g.TW;
        int d_tile = -1, d_j = ST_IT;           // tile being drained (-1: none), next store of it
        TileCoord d_tc = {0, 0, 0, 0};
        auto drain_begin = [&](int tile) {
            d_tile = tile;
            d_j = 0;
            d_tc = decode_tile<BN>(tile, g);
        };
        auto drain_store = [&]() {              // one wave-wide store; lanes outside the tensor are dropped by the range check
            if (d_tile < 0 || d_j >= ST_IT) return;              // wave-uniform: nothing left to drain
            const bool real = true;
            const int t = (sw + d_j * NSW) * ST_ROWS + lane / SPR;
            const int c16 = lane % SPR;
            const int th = (int)(((float)t + 0.5f) * g.inv_tw);
            const int tw = t - th * g.TW;
            const int p = d_tc.p0 + th, q = d_tc.q0 + tw;
            const int col = d_tc.k0 + c16 * 4;
            const bool ok = real & (t < npx) & (p < s.P) & (q < s.Q) & (col < s.K);
            const u32x4 v = lds[(staging_off >> 4) + t * SPR + (c16 ^ (t & (SPR < 16 ? SPR - 1 : 15)))];
            const uint32_t off = (uint32_t)(((d_tc.n * s.P + p) * s.Q + q) * s.K + col) * (uint32_t)sizeof(TO);
            store_piece<TO>(v, y_rsrc, ok ? off : y_bytes);
            ++d_j;
        };

        int tile = t_begin, tile_step = 0;
        for (int step = 0; step < steps; ++step) {
            __syncthreads();
            if (tile_step == 0 && tile > t_begin) drain_begin(tile - 1);     // deposited before this barrier
            // the previous tile leaves LDS SS stores per step, none in a tile's last step
            if (tile_step < steps_per_tile - 1) {
#pragma unroll
                for (int l = 0; l < SS; ++l) drain_store();
            }
            if (++tile_step == steps_per_tile) { tile_step = 0; ++tile; }
        }
        __syncthreads();                        // the last tile has been deposited
        drain_begin(t_end - 1);
        for (int j = 0; j < ST_IT; ++j) drain_store();
        return;
    }

    // =============================== compute waves ==============================================
    const int kh = wave / WAVES_P;              // K half of this wave (0 when KS == 1)
    const int wpos = wave - kh * WAVES_P;
    const int wave_m = wpos / WAVES_N, wave_n = wpos % WAVES_N;
    const int frow = lane & 31, fk = lane >> 5;
    const int npx = g.G * g.TH * g.TW;
    int a_base[MI];                             // patch pixel of each A-fragment row at tap (0, 0)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int t = (wave_m * MI + mi) * 32 + frow;
        const int tv = (int)(((float)t + 0.5f) * g.inv_tw);                 // row of the stacked tile
        const int tw = t - tv * g.TW;
        const int gi = g.G > 1 ? (int)(((float)tv + 0.5f) * g.inv_th) : 0;
        const int th = tv - gi * g.TH;
        a_base[mi] = t < npx ? ((gi * g.PH + th * s.stride) * g.PW + tw * s.stride) : 0;
    }
    int b_idx[NI][KI];                          // filter-fragment positions within a stage (16-byte units)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int row = (wave_n * NI + ni) * 32 + frow;
#pragma unroll
        for (int kk = 0; kk < KI; ++kk) b_idx[ni][kk] = row * CPR + swz<CPR>(row, kk * 2 + fk);
    }
    const bool vec_ok = (s.K & 3) == 0;
    // Byte address of the lane's 16 bytes of patch pixel pp for K slice 0: window pp / PPW (256 bytes, so the window
    // part of the address is a multiple of 256 and the slot part stays below 16), slot
    // ((pp % PPW)*CPR + l/32) ^ (window & wmask).  K slice kk is the slot xor 2*kk, i.e. the byte address xor (kk << 5):
    // one instruction per operand read.
    const char* lds_c = reinterpret_cast<const char*>(lds);
    auto operand_byte = [&](uint32_t patch_cur, uint32_t pp) __attribute__((always_inline)) {
        const uint32_t win = pp / (uint32_t)PPW;
        const uint32_t slot = ((pp % (uint32_t)PPW) * CPR + (uint32_t)fk) ^ (win & (uint32_t)wmask);
        return (patch_cur + win * 16u + slot) << 4;
    };

    // Epilogue of one tile for the fragments this wave owns.  The filter fragment is the MFMA's row
    // operand and the pixel fragment its column operand, so lane l holds block pixel 32*frag + l%32
    // and, in accumulator element v, filter 8*(v/4) + 4*(l/32) + v%4 of the 32-wide block: four
    // consecutive filters per group of four elements, stored as one 16-byte (fp32) or 8-byte
    // (16-bit) piece of the pixel's y row.  The stores are not waited for.
    auto store_tile = [&](int tile, floatx16 (&acc)[MI][NI]) __attribute__((always_inline)) {
        const TileCoord tc = decode_tile<BN>(tile, g);
        // The workgroup's LAST tile has nothing left to overlap its stores with, and the loader waves
        // end after its last step: once every compute wave is here LDS is free, and the fragments go
        // through wave-private staging areas so that each store covers whole 128-byte lines.  (A
        // barrier counts live waves only, so the ended loader waves do not take part.)
        if (SS == 0 && tile == t_end - 1 && vec_ok && (long long)g.G * g.TH * s.Q * s.K * (long long)sizeof(TO) < 0x7fffffffLL) {
            __syncthreads();
            if constexpr (KS == 2) {
                // partial sums of the upper K half: lane-linear 16-byte pieces behind the staging areas
                u32x4* red = lds + ((WAVES_C * kFragStageBytes) >> 4) + wpos * (MI * NI * 4 * 64) + lane;
                if (kh == 1) {
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                            for (int q = 0; q < 4; ++q) {
                                floatx4 v = {acc[mi][ni][4 * q], acc[mi][ni][4 * q + 1], acc[mi][ni][4 * q + 2], acc[mi][ni][4 * q + 3]};
                                red[((mi * NI + ni) * 4 + q) * 64] = __builtin_bit_cast(u32x4, v);
                            }
                }
                __syncthreads();
                if (kh == 1) return;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const floatx4 v = __builtin_bit_cast(floatx4, red[((mi * NI + ni) * 4 + q) * 64]);
                            acc[mi][ni][4 * q] += v[0]; acc[mi][ni][4 * q + 1] += v[1];
                            acc[mi][ni][4 * q + 2] += v[2]; acc[mi][ni][4 * q + 3] += v[3];
                        }
            }
            char* stg = reinterpret_cast<char*>(lds) + wave * kFragStageBytes;
            const size_t org = ((size_t)(tc.n * s.P + tc.p0) * s.Q + tc.q0) * s.K;
            const size_t rem = ((size_t)s.M * s.K - org) * sizeof(TO);
            const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + org, 0, rem > 0x7fffffffull ? 0x7fffffffu : (uint32_t)rem,
                                                                   kRsrcFlags);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
                    const int col0 = tc.k0 + (wave_n * NI + ni) * 32;
                    const bool pieces_ok = col0 + 4 * (lane & 7) + 3 < s.K;
                    store_frag_staged<TO>(stg, acc[mi][ni], lane, y_rsrc, pieces_ok, [&](int i) {
                        const int t = (wave_m * MI + mi) * 32 + i;
                        const int tv = (int)(((float)t + 0.5f) * g.inv_tw);
                        const int tw = t - tv * g.TW;
                        const int gi = g.G > 1 ? (int)(((float)tv + 0.5f) * g.inv_th) : 0;
                        const int th = tv - gi * g.TH;
                        const bool ok = (t < npx) & (tc.p0 + th < s.P) & (tc.q0 + tw < s.Q) & (tc.n + gi < s.N);
                        return ok ? (uint32_t)(((gi * s.P + th) * s.Q + tw) * s.K + col0) * (uint32_t)sizeof(TO) : 0x80000000u;
                    });
                }
            return;
        }
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            // (row, column) of the lane's pixel in the output block and its image within the tile: recomputed per tile
            // rather than kept in registers through the K loop
            int frow_v = frow;
            asm volatile("" : "+v"(frow_v));
            const int t = (wave_m * MI + mi) * 32 + frow_v;
            const int tv = (int)(((float)t + 0.5f) * g.inv_tw);
            const int o_tw = t - tv * g.TW;
            const int o_gi = g.G > 1 ? (int)(((float)tv + 0.5f) * g.inv_th) : 0;
            const int o_th = tv - o_gi * g.TH;
            const int p = tc.p0 + o_th, q = tc.q0 + o_tw, n = tc.n + o_gi;
            if (t < npx && p < s.P && q < s.Q && n < s.N) {
                TO* yrow = y + (size_t)((n * s.P + p) * s.Q + q) * s.K;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const int col = tc.k0 + (wave_n * NI + ni) * 32 + 8 * gq + 4 * fk;
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
    };

    if constexpr (PF != 0) {
        // ---- prefetching pipeline.  The K slices of a step form KG groups of KPG slices.  The operands of group g + 1 are read from LDS
        // before the MFMAs of group g are issued, across step boundaries too: the first group of
        // step i + 1 is read during step i.  The matrix pipe therefore never waits for an LDS read
        // after a barrier; in return the loaders keep one more filter stage complete.
        constexpr int KPG = KI >= 4 ? 2 : 1;        // slices per group
        constexpr int KG = KI / KPG;                // groups per step
        // read cursor: the step whose operands are fetched next
        int r_stage = 0, r_phase = 0, r_tr = 0, r_ts = 0;
        uint32_t a_byte[MI];                        // byte address of the step's pixel-fragment operand, K slice 0
        const u32x4* Bt = lds;
        auto point = [&]() __attribute__((always_inline)) {                        // operand addresses of the cursor's step
            const uint32_t patch_cur = (uint32_t)(r_phase & 1) * (g.patch_bytes >> 4);
            const int tap_off = (r_tr * g.PW + r_ts) * s.dil;
            Bt = lds + ((bstage_off + r_stage * BSTAGE_BYTES) >> 4);
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                a_byte[mi] = operand_byte(patch_cur, (uint32_t)(a_base[mi] + tap_off));
            }
        };
        auto advance = [&]() __attribute__((always_inline)) {      // branch-free: the step stays one scheduling region
            r_stage = r_stage + 1 == STB ? 0 : r_stage + 1;
            const int ts = r_ts + 1;
            const int wrap_s = ts == s.S ? 1 : 0;
            r_ts = wrap_s ? 0 : ts;
            const int tr = r_tr + wrap_s;
            const int wrap_r = tr == s.R ? 1 : 0;
            r_tr = wrap_r ? 0 : tr;
            r_phase += wrap_r;
        };
        frag_t af[2][KPG][MI], bfr[2][KPG][NI];
        auto read_group = [&](auto GK, auto BUF) __attribute__((always_inline)) {  // group GK of the cursor's step into register buffer BUF
            constexpr int gk = decltype(GK)::value, buf = decltype(BUF)::value;
#pragma unroll
            for (int k2 = 0; k2 < KPG; ++k2) {
                constexpr int j0 = gk * KPG;
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
                    af[buf][k2][mi] = *reinterpret_cast<const frag_t*>(lds_c + (a_byte[mi] ^ (uint32_t)((j0 + k2) << 5)));
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) bfr[buf][k2][ni] = __builtin_bit_cast(frag_t, Bt[b_idx[ni][j0 + k2]]);
            }
        };

        floatx16 acc[MI][NI];
        auto clear_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                    for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;
        };
        int tile = t_begin, tile_step = 0;
        auto one_step = [&](auto PAR) __attribute__((always_inline)) {             // PAR: register buffer that holds this step's first group
            constexpr int par = decltype(PAR)::value;
            __syncthreads();                        // the NEXT step's filter tile (and patch) has landed
            {
                // (the group number is a type: the register buffers must be indexed by constants)
                auto body = [&](auto GKT) __attribute__((always_inline)) {
                    constexpr int g0 = decltype(GKT)::value;
                    constexpr int cur = (par + g0) & 1, nxt = cur ^ 1;
                    if constexpr (g0 == KG - 1) {
                        advance();
                        point();
                        read_group(IntTag<0>{}, IntTag<nxt>{});
                    } else {
                        read_group(IntTag<g0 + 1>{}, IntTag<nxt>{});
                    }
#pragma unroll
                    for (int k2 = 0; k2 < KPG; ++k2)
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                            for (int ni = 0; ni < NI; ++ni)
                                acc[mi][ni] = Elem<T>::mfma32(bfr[cur][k2][ni], af[cur][k2][mi], acc[mi][ni]);
                    // A wave issues in order, so only instructions placed BETWEEN its MFMAs overlap with them.  The
                    // compiler's own interleaving of the next group's address arithmetic and LDS reads with this
                    // group's MFMAs measured 2-3 % faster than recipes of the form "one MFMA, n vector instructions,
                    // one LDS read" (n = 2, 3, 6, 8), so the order within a step is left to it.
                };
                body(IntTag<0>{});
                if constexpr (KG > 1) body(IntTag<1>{});
                if constexpr (KG > 2) body(IntTag<2>{});
                if constexpr (KG > 3) body(IntTag<3>{});
            }
            if (++tile_step == steps_per_tile) {
                store_tile(tile, acc);
                tile_step = 0;
                ++tile;
                clear_acc();
            }
        };
        static_assert(KG >= 1 && KG <= 4, "at most four groups per step");

        clear_acc();
        __syncthreads();                            // stage 0 and the first patch have landed
        point();
        read_group(IntTag<0>{}, IntTag<0>{});
        for (int step = 0; step < steps;) {
            one_step(IntTag<0>{});
            ++step;
            if constexpr ((KG & 1) != 0) {          // an odd number of groups flips the buffer parity per step
                if (step < steps) {
                    one_step(IntTag<1>{});
                    ++step;
                }
            }
        }
        return;
    }

    int stage = 0, phase = 0;
    for (int tile = t_begin; tile < t_end; ++tile) {
        floatx16 acc[MI][NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni)
#pragma unroll
                for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

        for (int ck = 0; ck < chunks; ++ck, ++phase) {
            const uint32_t patch_cur = (uint32_t)(phase & 1) * (g.patch_bytes >> 4);   // in 16-byte units
            int tap_r = 0, tap_s = 0;
            for (int t = 0; t < RS; ++t) {
                __syncthreads();                // this step's filter tile (and patch) has landed
                const int tap_off = (tap_r * g.PW + tap_s) * s.dil;
                const u32x4* Bt = lds + ((bstage_off + stage * BSTAGE_BYTES) >> 4);
                uint32_t a_byte[MI];
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) a_byte[mi] = operand_byte(patch_cur, (uint32_t)(a_base[mi] + tap_off));
                // operand fragments LDS -> registers and MFMAs, in KG groups of K slices: all reads of
                // a group are issued before its first MFMA, and the next group's reads follow that
                // group's MFMAs into the pipe
                constexpr int KG = KI >= 4 ? 2 : 1;     // groups per step
                constexpr int KPG = KI / KG;            // K slices per group
                static_assert(KS == 1 || KG == 2, "the K split takes one group each");
#pragma unroll
                for (int gk = 0; gk < KG; ++gk) {
                    if (KS == 2 && gk != kh) continue;      // uniform: the other half is the other wave's
                    frag_t af[KPG][MI], bfr[KPG][NI];
#pragma unroll
                    for (int k2 = 0; k2 < KPG; ++k2) {
                        const int kk = gk * KPG + k2;
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi)
                            af[k2][mi] = *reinterpret_cast<const frag_t*>(lds_c + (a_byte[mi] ^ (uint32_t)(kk << 5)));
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) bfr[k2][ni] = __builtin_bit_cast(frag_t, Bt[b_idx[ni][kk]]);
                    }
                    // All reads of the group before its first MFMA -- except for wave tiles of four fragments and
                    // for the K split, where letting the compiler start the MFMAs under the last reads measured
                    // 2-4 % faster (and 2-3 % slower for the two-fragment wave tiles).
                    if constexpr (!(KS == 2 || MI * NI >= 4)) __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int k2 = 0; k2 < KPG; ++k2)
#pragma unroll
                        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                            for (int ni = 0; ni < NI; ++ni)
                                acc[mi][ni] = Elem<T>::mfma32(bfr[k2][ni], af[k2][mi], acc[mi][ni]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                stage = stage + 1 == STB ? 0 : stage + 1;
                if (++tap_s == s.S) { tap_s = 0; ++tap_r; }
            }
        }

        // ---- the tile's epilogue: into the staging buffer for the store waves, or straight to y
        if (SS > 0) {
            // deposit: fp32 piece (pixel t, filters 4*c16 .. +3) at staging[t*SPR + (c16 ^ (t & 15))]
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int t = (wave_m * MI + mi) * 32 + frow;
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                    for (int gq = 0; gq < 4; ++gq) {
                        const int c16 = (wave_n * NI + ni) * 8 + 2 * gq + fk;
                        floatx4 v = {acc[mi][ni][4 * gq], acc[mi][ni][4 * gq + 1], acc[mi][ni][4 * gq + 2], acc[mi][ni][4 * gq + 3]};
                        lds[(staging_off >> 4) + t * SPR + (c16 ^ (t & (SPR < 16 ? SPR - 1 : 15)))] = __builtin_bit_cast(u32x4, v);
                    }
                }
            }
            continue;
        }
        store_tile(tile, acc);
    }
    if (SS > 0) __syncthreads();                // hands the last tile to the loader waves
}

// ---- host side ------------------------------------------------------------------------------------

struct PatchCfg {
    const char* name;
    int cb, waves_m, waves_n, mi, ni, stb, la, nld, ss, nsw, pf, ks;
    int bm() const { return waves_m * mi * 32; }
    int bn() const { return waves_n * ni * 32; }
    int waves() const { return waves_m * waves_n * ks + nld + nsw; }   // compute + loader + store waves
    // LDS after the patches, the filter ring and the sinks: output staging for the store waves
    long tail_bytes() const { return ss > 0 ? (long)bm() * bn() * 4 : 0; }
};

constexpr int kLdsLimit = 160 * 1024;

// Chooses the output block TH x TW (TH*TW <= BM) for one kernel configuration.  Cost model: MFMA
// work of all (padded) tiles plus the patch pixels that have to be brought into LDS.
bool plan_geometry(const ConvShape& s, const PatchCfg& c, PatchGeom* g) {
    const int BM = c.bm();
    if ((double)s.K * s.Kg * 4.0 >= 4294967296.0) return false;   // out-of-range filter offsets must not wrap (see filter_tile)
    // the K split adds its partial sums in the staged epilogue of a workgroup's only tile: whole 16-byte pieces
    if (c.ks == 2 && (s.K & 3) != 0) return false;
    if (c.ss > 0) {
        // the staged epilogue stores through a 32-bit buffer descriptor, needs K % 4 == 0 for whole
        // 16-byte pieces, and must get a tile out within the steps of the next one
        const int chunks = (s.C + c.cb - 1) / c.cb;
        const int st_it = BM / (64 / (c.bn() / 4)) / c.nsw;
        if ((s.K & 3) != 0 || (double)s.M * s.K * 4.0 >= 4294967296.0) return false;
        if ((long)c.ss * ((long)chunks * s.R * s.S - 1) < st_it) return false;
    }
    const int rpb = 64 / (c.cb / 8);
    const int RS = s.R * s.S;
    double best = 1e300;
    bool found = false;
    for (int tw = 1; tw <= s.Q && tw <= BM; ++tw) {
        int th = BM / tw;
        if (th > s.P) th = s.P;
        if (th < 1) continue;
        const int ph = (th - 1) * s.stride + (s.R - 1) * s.dil + 1;
        const int pw = (tw - 1) * s.stride + (s.S - 1) * s.dil + 1;
        const long npix = (long)ph * pw;
        const int per_pass = rpb * c.nld;
        const int a_blocks = (int)((npix + per_pass - 1) / per_pass);
        const long patch_bytes = (long)a_blocks * c.nld * 1024;
        const long staging = c.tail_bytes();
        const long lds = 2 * patch_bytes + (long)c.stb * c.bn() * c.cb * 2 + c.nld * 1024 + staging;
        if (lds > kLdsLimit) continue;
        // the next phase's patch must fit into the loads of the steps that may carry it
        if ((long)c.la * (RS - c.stb + 1) < a_blocks) continue;
        const long tiles = (long)((s.P + th - 1) / th) * ((s.Q + tw - 1) / tw);
        const double cost = (double)tiles * ((double)BM * RS + 4.0 * (double)npix);
        if (cost < best) {
            best = cost;
            found = true;
            g->TH = th; g->TW = tw; g->PH = ph; g->PW = pw; g->npix = (int)npix;
            g->tiles_h = (s.P + th - 1) / th; g->tiles_w = (s.Q + tw - 1) / tw;
            g->tiles_n = (s.K + c.bn() - 1) / c.bn();
            g->a_blocks = a_blocks;
            g->dph = per_pass / pw; g->dpw = per_pass % pw;
            g->patch_bytes = (int)patch_bytes;
            g->inv_tw = 1.0f / (float)tw;
        }
    }
    if (!found) return false;
    g->G = 1;
    g->inv_th = 1.0f / (float)g->TH;
    g->inv_ph = 1.0f / (float)g->PH;
    // A map that fits a tile at least twice (the 7 x 7 maps at the end of a network): several whole
    // images per tile, as many as the rows and LDS hold.  The filter tile of a step then serves all of
    // them, and the filter traffic per output, which is what binds these layers, drops accordingly.
    if (c.ss == 0 && g->TH == s.P && g->TW == s.Q) {
        const int per_pass = rpb * c.nld;
        for (int G = std::min(BM / (s.P * s.Q), s.N); G >= 2; --G) {
            const long npix = (long)G * g->PH * g->PW;
            const int a_blocks = (int)((npix + per_pass - 1) / per_pass);
            const long patch_bytes = (long)a_blocks * c.nld * 1024;
            const long lds = 2 * patch_bytes + (long)c.stb * c.bn() * c.cb * 2 + c.nld * 1024 + c.tail_bytes();
            if (lds > kLdsLimit || (long)c.la * (RS - c.stb + 1) < a_blocks) continue;
            if (per_pass / g->PW + 1 > g->PH) break;    // a patch load must not skip an image (the loader adds at most one)
            g->G = G;
            g->npix = (int)npix;
            g->a_blocks = a_blocks;
            g->patch_bytes = (int)patch_bytes;
            break;
        }
    }
    // (the staged epilogue addresses a tile's outputs with 31 bits)
    if (c.ks == 2 && (long long)g->G * g->TH * s.Q * s.K * 4LL >= 0x7fffffffLL) return false;
    return true;
}

template <typename T, typename TO, int CB, int WAVES_M, int WAVES_N, int MI, int NI, int STB, int LA, int NLD, int SS, int NSW,
          int PF, int KS>
hipError_t launch_cfg(const PatchCfg& c, const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    PatchGeom g;
    if (!plan_geometry(s, c, &g)) return hipErrorInvalidConfiguration;
    const int lds_bytes = 2 * g.patch_bytes + STB * c.bn() * CB * 2 + NLD * 1024 + (int)c.tail_bytes();
    auto kern = ipatch_kernel<T, TO, CB, WAVES_M, WAVES_N, MI, NI, STB, LA, NLD, SS, NSW, PF, KS>;
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    const long total = (long)((s.N + g.G - 1) / g.G) * g.tiles_h * g.tiles_w * g.tiles_n;
    if (total > 0x7fffffffL) return hipErrorInvalidConfiguration;
    // resident workgroups per compute unit for this LDS size (cached per kernel and size)
    static std::atomic<long long> occ_slot{-1};
    const int occ = cached_occupancy(occ_slot, (const void*)kern, c.waves() * 64, lds_bytes);
    int nwg = 1;
    g.total_tiles = (int)total;
    g.tiles_m = (int)(total / g.tiles_n);
    const long w_bytes = (long)s.K * s.Kg * 2, x_bytes = (long)s.N * s.H * s.W * s.C * 2;
    g.n_slow = (g.tiles_n > 1 && w_bytes >= (2L << 20) && w_bytes > x_bytes) ? 1 : 0;
    const int cap = call_max_workgroups();
    if (KS == 2) {
        g.tiles_per_wg = 1;                     // the partial sums meet in LDS the loaders no longer use
        nwg = (int)total;
    } else if (cap > 0) {
        split_tiles(total, cap, 1, &g.tiles_per_wg, &nwg);
    } else {
        split_tiles(total, device_cus(), occ, &g.tiles_per_wg, &nwg);
    }
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(c.waves() * 64), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y, s, g);
    return hipGetLastError();
}

//   name                                  CB  WM WN MI NI STB LA NLD SS NSW PF
// (compute + loader [+ store] waves; SS > 0: output staged in LDS and drained by NSW store waves;
//  PF: operands of the next group of K slices are read before the current group's MFMAs; KS = 2: two compute waves
//  per tile position, one K half each: "4x2")
#define ICONV_PATCH_VARIANTS(X)                                                              \
    X(kP128x64, "p128x64_c64_w32x64_s3_4+4", 64, 4, 1, 1, 2, 3, 1, 4, 0, 0, 0, 1)                \
    X(kP256x128, "p256x128_c64_w64x64_s3_8+4", 64, 4, 2, 2, 2, 3, 2, 4, 0, 0, 0, 1)              \
    X(kP256x64, "p256x64_c64_w32x64_s3_8+4", 64, 8, 1, 1, 2, 3, 2, 4, 0, 0, 0, 1)                \
    X(kP64x64, "p64x64_c64_w32x32_s3_4+4", 64, 2, 2, 1, 1, 3, 1, 4, 0, 0, 0, 1)                  \
    X(kP64x128, "p64x128_c64_w32x64_s3_4+4", 64, 2, 2, 1, 2, 3, 1, 4, 0, 0, 0, 1)                \
    X(kP128x64Staged, "p128x64_c64_w32x64_s3_4+4+2", 64, 4, 1, 1, 2, 3, 2, 4, 2, 2, 0, 1)        \
    X(kP256x128Pf, "p256x128_c64_w64x64_s3_8+4_pf", 64, 4, 2, 2, 2, 3, 2, 4, 0, 0, 1, 1)         \
    X(kP64x128Pf, "p64x128_c64_w32x64_s4_4+4_pf", 64, 2, 2, 1, 2, 4, 1, 4, 0, 0, 1, 1)           \
    X(kP64x128C128, "p64x128_c128_w32x64_s3_4+4", 128, 2, 2, 1, 2, 3, 1, 4, 0, 0, 0, 1)      \
    X(kP64x128C128K2, "p64x128_c128_w32x64_s3_4x2+4", 128, 2, 2, 1, 2, 3, 1, 4, 0, 0, 0, 2)

#define X_CFG(i, name, cb, wm, wn, mi, ni, stb, la, nld, ss, nsw, pf, ks) {name, cb, wm, wn, mi, ni, stb, la, nld, ss, nsw, pf, ks},
const PatchCfg kPatchCfgs[] = {ICONV_PATCH_VARIANTS(X_CFG)};
#undef X_CFG
static_assert(sizeof(kPatchCfgs) / sizeof(kPatchCfgs[0]) == kNumPatch, "one configuration per kernel");

template <typename T, typename TO>
hipError_t launch_patch_t(int v, const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    switch (v) {
#define X_CASE(i, name, cb, wm, wn, mi, ni, stb, la, nld, ss, nsw, pf, ks) \
    case i: return launch_cfg<T, TO, cb, wm, wn, mi, ni, stb, la, nld, ss, nsw, pf, ks>(kPatchCfgs[i], x, w, y, s, st);
        ICONV_PATCH_VARIANTS(X_CASE)
#undef X_CASE
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

int patch_num_variants() { return kNumPatch; }
const char* patch_variant_name(int v) { return kPatchCfgs[v].name; }

bool patch_supported(const ConvShape& s, int v) {
    if (v < 0 || v >= kNumPatch || (s.C % 8) != 0) return false;
    PatchGeom g;
    return plan_geometry(s, kPatchCfgs[v], &g);
}

hipError_t launch_patch(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v,
                        hipStream_t st) {
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_patch_t<bf16_t, float>(v, x, w, y, s, st);
        return launch_patch_t<bf16_t, bf16_t>(v, x, w, y, s, st);
    }
    if (out_t == OUT_F32) return launch_patch_t<f16_t, float>(v, x, w, y, s, st);
    return launch_patch_t<f16_t, f16_t>(v, x, w, y, s, st);
}

}  // namespace iconv

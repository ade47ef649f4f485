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
// BN filters), no atomics.
#include <atomic>

#include "iconv_common.h"
#include "iconv_device.h"

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
    int patch_bufs;      // 2 when the layer has several channel chunks (double buffer), else 1
    float inv_tw;        // 1 / TW
};

// Patch swizzle.  The patch is an array of 256-byte windows (all 64 LDS banks), each holding
// PPW = 16/CPR pixels of CPR 16-byte chunks.  Chunk c of pixel pp has logical slot
// (pp % PPW)*CPR + c in window pp / PPW and lives at physical slot  logical ^ (window & 15).
// An MFMA operand read has its 16 consecutive lanes on 16 pixels that are `stride` apart, same
// chunk: XOR-ing the window number into all four slot bits spreads those over the 16 slots for
// stride 1 (at most one clash when the run starts on an odd pixel) and for stride 2.
//
// Wave roles.  The workgroup has WAVES_M*WAVES_N compute waves and NLD loader waves.  Loader waves
// only issue the global -> LDS loads (their address arithmetic then overlaps the compute waves'
// MFMAs instead of delaying them); compute waves only read LDS and issue MFMAs.  All waves meet
// at one barrier per K step.
template <typename T, typename TO, int CB, int WAVES_M, int WAVES_N, int MI, int NI, int STB, int LA, int NLD>
__global__ void __launch_bounds__((WAVES_M * WAVES_N + NLD) * 64)
ipatch_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const PatchGeom g) {
    constexpr int WAVES_C = WAVES_M * WAVES_N;  // compute waves
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
    static_assert((STB - 2) * B_IT + (STB - 1) * LA < 64, "too many loads in flight for vmcnt");
    typedef typename Elem<T>::frag frag_t;

    extern __shared__ u32x4 lds[];   // [patch 0][patch 1 if needed][STB filter stages][1 KiB sink per loader wave]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    int tile = xcd_remap(blockIdx.x, gridDim.x);
    const int tile_n = tile % g.tiles_n; tile /= g.tiles_n;
    const int tile_w = tile % g.tiles_w; tile /= g.tiles_w;
    const int tile_h = tile % g.tiles_h;
    const int n = tile / g.tiles_h;
    const int p0 = tile_h * g.TH, q0 = tile_w * g.TW, k0 = tile_n * BN;

    const int RS = s.R * s.S;
    const int chunks = (s.C + CB - 1) / CB;
    const int steps = chunks * RS;
    const uint32_t bstage_off = (uint32_t)(g.patch_bufs * g.patch_bytes);   // byte offset of the filter ring

    if (wave >= WAVES_C) {
        // =========================== loader waves ===========================================
        const int lw = wave - WAVES_C;
        const int h_base = p0 * s.stride - s.pad, w_base = q0 * s.stride - s.pad;
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
        const int a_slot = (lane & 15) ^ (a_win0 & 15);
        const int a_lc = (a_slot % CPR) * 8;    // first channel (within a chunk) this lane fetches
        const int a_pp0 = a_win0 * PPW + a_slot / CPR;
        const int a_ph0 = a_pp0 / g.PW;
        const int a_pw0 = a_pp0 - a_ph0 * g.PW;
        int a_ph, a_pw, a_j;                    // running state within one channel chunk
        auto patch_reset = [&]() { a_ph = a_ph0; a_pw = a_pw0; a_j = 0; };
        // one patch load of channel chunk `c0` into patch buffer `buf` (or a no-op load into the sink)
        auto patch_load = [&](int buf, int c0, bool live) {
            const int h = h_base + a_ph, ww = w_base + a_pw;
            const bool real = live && a_j < g.a_blocks;          // wave-uniform
            const bool ok = real & (a_ph < g.PH) & ((unsigned)h < (unsigned)s.H) & ((unsigned)ww < (unsigned)s.W) &
                            ((c0 + a_lc) < s.C);
            const uint32_t off = (uint32_t)(((n * s.H + h) * s.W + ww) * s.C + c0 + a_lc) * 2u;
            const uint32_t dst = real ? lds_base + (uint32_t)buf * g.patch_bytes + (uint32_t)(lw + a_j * NLD) * 1024u : sink;
            dma16(x_rsrc, ok ? off : x_bytes, (uint32_t)__builtin_amdgcn_readfirstlane((int)dst));
            a_pw += g.dpw;
            const int wrap = a_pw >= g.PW ? 1 : 0;
            a_pw -= wrap ? g.PW : 0;
            a_ph += g.dph + wrap;
            ++a_j;
        };

        // ---- filter-tile loads (one BN x CB tile per step)
        const int pc = lane % CPR, lr = lane / CPR;
        uint32_t b_off[B_IT];
        bool b_ok[B_IT];
#pragma unroll
        for (int j = 0; j < B_IT; ++j) {
            const int row = (lw + j * NLD) * RPB + lr;
            const int ch = swz<CPR>(row, pc) * 8;
            b_ok[j] = (k0 + row) < s.K;
            b_off[j] = (uint32_t)((k0 + row) * s.Kg + ch) * 2u;
        }
        const bool ragged_c = (s.C % CB) != 0;
        int lr_ = 0, ls_ = 0, lc0 = 0;          // tap (lr_, ls_) of channel chunk lc0 to load next
        auto filter_load = [&](int stage, bool live) {
            const uint32_t delta = (uint32_t)((lr_ * s.S + ls_) * s.C + lc0) * 2u;
#pragma unroll
            for (int j = 0; j < B_IT; ++j) {
                bool ok = live & b_ok[j];
                if (ragged_c) {
                    const int row = (lw + j * NLD) * RPB + lr;
                    ok = ok & ((lc0 + swz<CPR>(row, pc) * 8) < s.C);
                }
                dma16(w_rsrc, ok ? b_off[j] + delta : w_bytes,
                      bstage_base + (uint32_t)(stage * BSTAGE_BYTES + (lw + j * NLD) * 1024));
            }
            if (++ls_ == s.S) {
                ls_ = 0;
                if (++lr_ == s.R) { lr_ = 0; lc0 += CB; }
            }
        };

        // prologue: the whole patch of chunk 0, then what the STB-1 steps before the first one would
        // have issued (their filter tiles; no-op loads in place of patch slices), so that the
        // steady-state wait count holds from the first step on.  Loads complete in issue order, so
        // the first step's wait for its filter tile also covers the patch.
        patch_reset();
        for (int j = 0; j < g.a_blocks; ++j) patch_load(0, 0, true);
        patch_reset();
#pragma unroll
        for (int j = 0; j < STB - 1; ++j) {
            filter_load(j, j < steps);
#pragma unroll
            for (int l = 0; l < LA; ++l) dma16(x_rsrc, x_bytes, sink);
        }
        int fill = STB - 1, step = 0;
        for (int ck = 0; ck < chunks; ++ck) {
            const bool next_chunk = ck + 1 < chunks;
            for (int t = 0; t < RS; ++t, ++step) {
                // Everything issued after this step's filter tile may stay in flight: STB-2 later
                // filter tiles and STB-1 groups of patch loads.
                wait_vmcnt<(STB - 2) * B_IT + (STB - 1) * LA>();
                __syncthreads();
                filter_load(fill, step + STB - 1 < steps);
                // The next chunk's patch arrives LA loads per step; the last STB-1 steps of a chunk
                // carry no-op loads only, so the patch is complete once the next chunk's first step
                // has waited.
#pragma unroll
                for (int l = 0; l < LA; ++l) patch_load((ck + 1) & 1, (ck + 1) * CB, next_chunk && t <= RS - STB);
                fill = fill + 1 == STB ? 0 : fill + 1;
            }
            patch_reset();
        }
        wait_vmcnt<0>();
        return;
    }

    // =============================== compute waves ==============================================
    const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
    const int frow = lane & 31, fk = lane >> 5;
    const int npx = g.TH * g.TW;
    int a_base[MI];                             // patch pixel of each A-fragment row at tap (0, 0)
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int t = (wave_m * MI + mi) * 32 + frow;
        const int th = (int)(((float)t + 0.5f) * g.inv_tw);
        const int tw = t - th * g.TW;
        a_base[mi] = t < npx ? (th * g.PW + tw) * s.stride : 0;
    }
    int b_idx[NI][KI];                          // filter-fragment positions within a stage (16-byte units)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
        const int row = (wave_n * NI + ni) * 32 + frow;
#pragma unroll
        for (int kk = 0; kk < KI; ++kk) b_idx[ni][kk] = row * CPR + swz<CPR>(row, kk * 2 + fk);
    }

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    int stage = 0;
    for (int ck = 0; ck < chunks; ++ck) {
        const uint32_t patch_cur = (uint32_t)(ck & 1) * (g.patch_bytes >> 4);   // in 16-byte units
        int tap_r = 0, tap_s = 0;
        for (int t = 0; t < RS; ++t) {
            __syncthreads();                    // this step's filter tile (and patch) has landed
            const int tap_off = (tap_r * g.PW + tap_s) * s.dil;
            const u32x4* Bt = lds + ((bstage_off + stage * BSTAGE_BYTES) >> 4);
            int a_win[MI], a_sx[MI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int pp = a_base[mi] + tap_off;
                a_win[mi] = patch_cur + (pp / PPW) * 16;              // 256-byte window of this pixel
                a_sx[mi] = ((pp % PPW) * CPR + fk) ^ ((pp / PPW) & 15);
            }
            // operand fragments LDS -> registers and MFMAs, in KG groups of K slices: all reads of a
            // group are issued before its first MFMA, and the next group's reads follow that group's
            // MFMAs into the pipe
            constexpr int KG = KI >= 4 ? 2 : 1;     // groups per step
            constexpr int KPG = KI / KG;            // K slices per group
#pragma unroll
            for (int gk = 0; gk < KG; ++gk) {
                frag_t af[KPG][MI], bfr[KPG][NI];
#pragma unroll
                for (int k2 = 0; k2 < KPG; ++k2) {
                    const int kk = gk * KPG + k2;
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi) af[k2][mi] = __builtin_bit_cast(frag_t, lds[a_win[mi] + (a_sx[mi] ^ (kk * 2))]);
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) bfr[k2][ni] = __builtin_bit_cast(frag_t, Bt[b_idx[ni][kk]]);
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int k2 = 0; k2 < KPG; ++k2)
#pragma unroll
                    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                        for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Elem<T>::mfma32(bfr[k2][ni], af[k2][mi], acc[mi][ni]);
                __builtin_amdgcn_sched_barrier(0);
            }
            stage = stage + 1 == STB ? 0 : stage + 1;
            if (++tap_s == s.S) { tap_s = 0; ++tap_r; }
        }
    }

    // ---- epilogue.  The filter fragment is the MFMA's row operand and the pixel fragment its
    // column operand, so lane l holds tile pixel 32*frag + l%32 and, in accumulator element v,
    // filter 8*(v/4) + 4*(l/32) + v%4 of the 32-wide block: four consecutive filters per group of
    // four elements, stored as one 16-byte (fp32) or 8-byte (16-bit) piece of the pixel's y row.
    const bool vec_ok = (s.K & 3) == 0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int t = (wave_m * MI + mi) * 32 + frow;
        const int th = (int)(((float)t + 0.5f) * g.inv_tw);
        const int tw = t - th * g.TW;
        const int p = p0 + th, q = q0 + tw;
        if (t < npx && p < s.P && q < s.Q) {
            TO* yrow = y + (size_t)((n * s.P + p) * s.Q + q) * s.K;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int col = k0 + (wave_n * NI + ni) * 32 + 8 * gq + 4 * fk;
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
}

// ---- host side ------------------------------------------------------------------------------------

struct PatchCfg {
    const char* name;
    int cb, waves_m, waves_n, mi, ni, stb, la, nld;
    int bm() const { return waves_m * mi * 32; }
    int bn() const { return waves_n * ni * 32; }
    int waves() const { return waves_m * waves_n + nld; }   // compute + loader waves
};

constexpr int kLdsLimit = 160 * 1024;

// Chooses the output block TH x TW (TH*TW <= BM) for one kernel configuration.  Cost model: MFMA
// work of all (padded) tiles plus the patch pixels that have to be brought into LDS.
bool plan_geometry(const ConvShape& s, const PatchCfg& c, PatchGeom* g) {
    const int BM = c.bm();
    const int rpb = 64 / (c.cb / 8);
    const int RS = s.R * s.S;
    const int chunks = (s.C + c.cb - 1) / c.cb;
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
        const int bufs = chunks > 1 ? 2 : 1;
        const long lds = bufs * patch_bytes + (long)c.stb * c.bn() * c.cb * 2 + c.nld * 1024;
        if (lds > kLdsLimit) continue;
        // a later chunk's patch must fit into the loads of the steps that may carry it
        if (chunks > 1 && (long)c.la * (RS - c.stb + 1) < a_blocks) continue;
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
            g->patch_bufs = bufs;
            g->inv_tw = 1.0f / (float)tw;
        }
    }
    return found;
}

template <typename T, typename TO, int CB, int WAVES_M, int WAVES_N, int MI, int NI, int STB, int LA, int NLD>
hipError_t launch_cfg(const PatchCfg& c, const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    PatchGeom g;
    if (!plan_geometry(s, c, &g)) return hipErrorInvalidConfiguration;
    const int lds_bytes = g.patch_bufs * g.patch_bytes + STB * c.bn() * CB * 2 + NLD * 1024;
    auto kern = ipatch_kernel<T, TO, CB, WAVES_M, WAVES_N, MI, NI, STB, LA, NLD>;
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsLimit);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    const long grid = (long)s.N * g.tiles_h * g.tiles_w * g.tiles_n;
    if (grid > 0x7fffffffL) return hipErrorInvalidConfiguration;
    hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(c.waves() * 64), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y,
                       s, g);
    return hipGetLastError();
}

//   name                               CB  WM WN MI NI STB LA NLD   (compute waves + loader waves)
#define ICONV_PATCH_VARIANTS(X)                                          \
    X(0, "p256x64_c64_w64x64_s3_4+4", 64, 4, 1, 2, 2, 3, 2, 4)           \
    X(1, "p128x64_c64_w32x64_s3_4+4", 64, 4, 1, 1, 2, 3, 1, 4)           \
    X(2, "p128x128_c64_w64x64_s3_4+4", 64, 2, 2, 2, 2, 3, 2, 4)          \
    X(3, "p256x128_c64_w64x64_s3_8+4", 64, 4, 2, 2, 2, 3, 2, 4)          \
    X(4, "p128x128_c32_w64x64_s4_4+4", 32, 2, 2, 2, 2, 4, 2, 4)          \
    X(5, "p256x64_c64_w32x64_s3_8+4", 64, 8, 1, 1, 2, 3, 2, 4)           \
    X(6, "p256x64_c64_w64x32_s3_8+4", 64, 4, 2, 2, 1, 3, 2, 4)           \
    X(7, "p64x64_c64_w32x32_s3_4+4", 64, 2, 2, 1, 1, 3, 1, 4)            \
    X(8, "p64x128_c64_w32x64_s3_4+4", 64, 2, 2, 1, 2, 3, 1, 4)           \
    X(9, "p128x256_c32_w64x64_s3_8+4", 32, 2, 4, 2, 2, 3, 1, 4)          \
    X(10, "p256x128_c64_w128x64_s3_4+4", 64, 2, 2, 4, 2, 3, 3, 4)

#define X_CFG(i, name, cb, wm, wn, mi, ni, stb, la, nld) {name, cb, wm, wn, mi, ni, stb, la, nld},
const PatchCfg kPatchCfgs[] = {ICONV_PATCH_VARIANTS(X_CFG)};
#undef X_CFG
constexpr int kNumPatch = sizeof(kPatchCfgs) / sizeof(kPatchCfgs[0]);

template <typename T, typename TO>
hipError_t launch_patch_t(int v, const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    switch (v) {
#define X_CASE(i, name, cb, wm, wn, mi, ni, stb, la, nld) \
    case i: return launch_cfg<T, TO, cb, wm, wn, mi, ni, stb, la, nld>(kPatchCfgs[i], x, w, y, s, st);
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

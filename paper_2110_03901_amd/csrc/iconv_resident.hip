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
// Waves.  Four compute waves (one per SIMD) each own MF*16 consecutive pixels of the block and
// all 64 filters: MF x 4 accumulator tiles of the 16x16x32 MFMA, so one K step reads MF + 4
// operand fragments for 4*MF MFMAs.  Output blocks of MF*64 pixels tile feature maps whose
// width is a multiple of 7 or 8 without padding rows of the MFMA.  Two loader waves issue the
// global -> LDS loads of the next channel slice (of this block or the next) while a slice is
// computed; the loads of a workgroup's very first slice are shared by all six waves.
//
// LDS.  Patch slice and filter slice use the same layout: rows (a pixel, or a filter) of 64
// bytes = four 16-byte chunks of 8 channels, chunk c of row i stored at chunk c ^ ((i >> 2) & 3).
// An operand read has 16 consecutive lanes on 16 consecutive rows and the same chunk, which
// then fall on 16 different 16-byte positions of the 256-byte bank window.
#include <atomic>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

constexpr int kResWaves = 4;         // compute waves
constexpr int kResLoaders = 2;       // loader waves
constexpr int kResBN = 64;           // filters per workgroup
constexpr int kResStage = 2048;      // output staging bytes per compute wave

struct ResGeom {
    int TH, TW;          // output block
    int PH, PW;          // input patch
    int npix;            // PH * PW
    int tiles_h, tiles_w;
    int total_tiles;
    int tiles_base, tiles_rem;   // workgroup i owns tiles_base (+1 if i < tiles_rem) consecutive blocks
    int KS;              // channel slices of 32
    int NR;              // patch regions in LDS: max(KS, 2)
    int slice_bytes;     // LDS bytes of one patch region (multiple of 1024)
    int w_bytes;         // LDS bytes of the filters: R*S*C*128
    int patch_loads;     // wave-wide loads per patch slice
    float inv_tw, inv_pw, inv_s;
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

template <typename T> struct Mfma16;
template <> struct Mfma16<bf16_t> {
    static __device__ __forceinline__ floatx4 run(bf16x8 a, bf16x8 b, floatx4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Mfma16<f16_t> {
    static __device__ __forceinline__ floatx4 run(f16x8 a, f16x8 b, floatx4 c) {
        return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
    }
};

template <typename T, typename TO, int MF>
__global__ void __launch_bounds__((kResWaves + kResLoaders) * 64)
ires_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const ResGeom g) {
    typedef typename Elem<T>::frag frag_t;
    constexpr int NWAVES = kResWaves + kResLoaders;
    // [filters: (slice, tap, filter 0..63) x 64 B][NR patch regions: pixel x 64 B][staging: 2 KiB per compute wave]
    extern __shared__ u32x4 lds[];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int wg = xcd_remap(blockIdx.x, gridDim.x);
    const int t_begin = wg * g.tiles_base + min(wg, g.tiles_rem);
    const int t_end = t_begin + g.tiles_base + (wg < g.tiles_rem ? 1 : 0);
    const int RS = s.R * s.S;
    const int phases = (t_end - t_begin) * g.KS;             // (block, channel slice) pairs of this workgroup
    if (phases <= 0) return;

    // ---- global -> LDS loads of one phase, split over `nparts` waves (this wave is `part`).
    // Wave-wide load j of a slice fills rows 16j .. 16j+15: lane l fetches row 16j + l/4, the
    // logical chunk that lives at physical chunk l%4 of that row.
    const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * s.C * 2u;
    const uint32_t w_bytes = (uint32_t)s.K * s.Kg * 2u;
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
    const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds;
    const int l_row = lane >> 2, l_pc = lane & 3;
    auto issue_loads = [&](int phase, int part, int nparts) {
        const int ks = phase % g.KS;
        int in_flight = 0;
        if (phase < g.KS) {
            // filters of this slice (first block only): load j covers tap j/4, filters 16*(j%4) + l/4
            for (int j = part; j < RS * 4; j += nparts) {
                const int f = (j & 3) * 16 + l_row;
                const int chunk = l_pc ^ ((f >> 2) & 3);
                const uint32_t off = (uint32_t)(f * s.Kg + (j >> 2) * s.C + ks * 32 + chunk * 8) * 2u;
                dma16(w_rsrc, f < s.K ? off : w_bytes,
                      (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_base + (uint32_t)((ks * RS * 4 + j) * 1024))));
                if (++in_flight == 24) { wait_vmcnt<16>(); in_flight = 16; }
            }
        }
        const ResTile tc = res_decode(t_begin + phase / g.KS, g);
        const int h_org = tc.p0 * s.stride - s.pad, w_org = tc.q0 * s.stride - s.pad;
        const uint32_t region = lds_base + (uint32_t)g.w_bytes + (uint32_t)(phase % g.NR) * (uint32_t)g.slice_bytes;
        for (int j = part; j < g.patch_loads; j += nparts) {
            const int pp = j * 16 + l_row;
            const int ph = (int)(((float)pp + 0.5f) * g.inv_pw);
            const int pw = pp - ph * g.PW;
            const int h = h_org + ph, ww = w_org + pw;
            const bool ok = (pp < g.npix) & ((unsigned)h < (unsigned)s.H) & ((unsigned)ww < (unsigned)s.W);
            const int chunk = l_pc ^ ((pp >> 2) & 3);
            const uint32_t off = (uint32_t)(((tc.n * s.H + h) * s.W + ww) * s.C + ks * 32 + chunk * 8) * 2u;
            dma16(x_rsrc, ok ? off : x_bytes, (uint32_t)__builtin_amdgcn_readfirstlane((int)(region + (uint32_t)(j * 1024))));
            if (++in_flight == 24) { wait_vmcnt<16>(); in_flight = 16; }
        }
    };

    issue_loads(0, wave, NWAVES);               // the first phase's loads are shared by all waves

    if (wave >= kResWaves) {
        // =========================== loader waves ===========================================
        const int lw = wave - kResWaves;
        for (int p = 0; p < phases; ++p) {
            wait_vmcnt<0>();
            __syncthreads();                    // phase p is in LDS; every wave has finished phase p - 1
            // region (p + 1) % NR was last read in phase p + 1 - NR <= p - 1
            if (p + 1 < phases) issue_loads(p + 1, lw, kResLoaders);
        }
        return;
    }

    // =============================== compute waves ==============================================
    const int l16 = lane & 15, lc = lane >> 4, lc16 = lc << 4;
    const int npx = g.TH * g.TW;
    const char* lds_b = reinterpret_cast<const char*>(lds);
    int a_pix[MF];                              // patch pixel of the lane's output pixel at tap (0, 0), per fragment
#pragma unroll
    for (int mf = 0; mf < MF; ++mf) {
        const int t = (wave * MF + mf) * 16 + l16;
        const int th = (int)(((float)t + 0.5f) * g.inv_tw);
        const int tw = t - th * g.TW;
        a_pix[mf] = t < npx ? (th * g.PW + tw) * s.stride : 0;
    }
    // filter fragment nf of (slice, tap): filter 16*nf + l%16, chunk l/16
    const uint32_t b_lane = (uint32_t)(l16 * 64 + ((lc ^ (l16 >> 2)) << 4));
    // output staging, 16 pixels x 32 filters at a time: piece c (16 bytes) of pixel i at i*128 + ((c ^ ((i >> 1) & 7)) << 4)
    char* stg = reinterpret_cast<char*>(lds) + g.w_bytes + g.NR * g.slice_bytes + wave * kResStage;
    const uint32_t sw0 = (uint32_t)(l16 * 128 + ((lc ^ ((l16 >> 1) & 7)) << 4));        // pieces lc (first filter block), lc + 4
    const uint32_t sw1 = (uint32_t)(l16 * 128 + (((lc + 4) ^ ((l16 >> 1) & 7)) << 4));
    const int l8 = lane >> 3, c8 = lane & 7;
    const uint32_t sr0 = (uint32_t)(l8 * 128 + ((c8 ^ ((l8 >> 1) & 7)) << 4));          // pixel l/8 (+8), piece l%8
    const uint32_t sr1 = (uint32_t)((l8 + 8) * 128 + ((c8 ^ (((l8 + 8) >> 1) & 7)) << 4));
    const size_t y_elems = (size_t)s.M * s.K;

    wait_vmcnt<0>();                            // this wave's share of the first phase's loads
    floatx4 acc[MF][4];
    for (int p = 0; p < phases; ++p) {
        __syncthreads();                        // phase p is in LDS
        const int ks = p % g.KS;
        const char* pa = lds_b + g.w_bytes + (p % g.NR) * g.slice_bytes;
        const char* pb = lds_b + b_lane + ks * RS * 4096;
        frag_t af[MF], b0[4], b1[4];

        auto tap_offset = [&](int t) {
            const int r = (int)(((float)t + 0.5f) * g.inv_s);
            return (r * g.PW + (t - r * s.S)) * s.dil;
        };
        auto fetch_a = [&](int tap_off, int mf) {
            const int pix = a_pix[mf] + tap_off;
            return *reinterpret_cast<const frag_t*>(pa + pix * 64 + (((pix << 2) & 0x30) ^ lc16));
        };
        // One tap: the filter fragments of the next tap are read into the other B set first, and each
        // pixel fragment is re-read for the next tap as soon as its four MFMAs have been issued, so
        // the LDS reads of tap t + 1 run under the MFMAs of tap t with one A set and two B sets.
        // (Past the last tap the reads repeat it: unconditional, and harmless.)
        auto step = [&](int t_next, const frag_t (&bc)[4], frag_t (&bn)[4], bool first) {
            const int off_next = tap_offset(t_next);
#pragma unroll
            for (int nf = 0; nf < 4; ++nf) bn[nf] = *reinterpret_cast<const frag_t*>(pb + t_next * 4096 + nf * 1024);
#pragma unroll
            for (int mf = 0; mf < MF; ++mf) {
                if (first) {
                    const floatx4 z = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int nf = 0; nf < 4; ++nf) acc[mf][nf] = Mfma16<T>::run(bc[nf], af[mf], z);
                } else {
#pragma unroll
                    for (int nf = 0; nf < 4; ++nf) acc[mf][nf] = Mfma16<T>::run(bc[nf], af[mf], acc[mf][nf]);
                }
                af[mf] = fetch_a(off_next, mf);
            }
        };
        const int t_last = RS - 1;
#pragma unroll
        for (int nf = 0; nf < 4; ++nf) b0[nf] = *reinterpret_cast<const frag_t*>(pb + nf * 1024);
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) af[mf] = fetch_a(0, mf);
        for (int t = 0; t < RS; t += 2) {
            step(min(t + 1, t_last), b0, b1, ks == 0 && t == 0);
            if (t + 1 < RS) step(min(t + 2, t_last), b1, b0, false);
        }
        if (ks + 1 < g.KS) continue;

        // ---- epilogue of the block.  The filters are the MFMA's row operand: lane l holds pixel
        // l%16 of fragment mf and filters 16*nf + 4*(l/16) .. +3 in acc[mf][nf].  Two filter blocks
        // at a time go through the wave's staging area (in-order LDS, no wait needed in between)
        // and leave as 16-byte pieces, 8 lanes per pixel = one 128-byte line of the y row.
        const ResTile tc = res_decode(t_begin + p / g.KS, g);
        const size_t org = ((size_t)(tc.n * s.P + tc.p0) * s.Q + tc.q0) * s.K;
        const size_t rem = (y_elems - org) * sizeof(TO);
        const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + org, 0, rem > 0xffffffffull ? 0xffffffffu : (uint32_t)rem,
                                                               kRsrcFlags);
#pragma unroll
        for (int mf = 0; mf < MF; ++mf) {
            u32x4 out[2][2];
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                __builtin_amdgcn_wave_barrier();
                *reinterpret_cast<floatx4*>(stg + sw0) = acc[mf][2 * h];
                *reinterpret_cast<floatx4*>(stg + sw1) = acc[mf][2 * h + 1];
                __builtin_amdgcn_wave_barrier();
                out[h][0] = *reinterpret_cast<const u32x4*>(stg + sr0);
                out[h][1] = *reinterpret_cast<const u32x4*>(stg + sr1);
            }
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const int t = (wave * MF + mf) * 16 + 8 * j + l8;
                const int th = (int)(((float)t + 0.5f) * g.inv_tw);
                const int tw = t - th * g.TW;
                const bool pix_ok = (t < npx) & (tc.p0 + th < s.P) & (tc.q0 + tw < s.Q);
                const uint32_t off = (uint32_t)((th * s.Q + tw) * s.K + 4 * c8) * (uint32_t)sizeof(TO);
#pragma unroll
                for (int h = 0; h < 2; ++h)
                    if (pix_ok && h * 32 + 4 * c8 + 3 < s.K)
                        store_piece<TO>(out[h][j], y_rsrc, off + (uint32_t)(h * 32 * sizeof(TO)));
            }
        }
    }
}

constexpr int kResLdsLimit = 160 * 1024;

// Chooses the output block TH x TW (TH*TW <= 64*MF) for a fragment count MF.  Cost model as for
// the patch-reuse kernels: MFMA work of all (padded) blocks plus the patch pixels brought into LDS.
bool plan_res(const ConvShape& s, int MF, ResGeom* g, double* cost_out) {
    if ((s.C % 32) != 0 || (s.K & 3) != 0 || s.K > kResBN) return false;
    const int BM = kResWaves * MF * 16;
    const int RS = s.R * s.S;
    const long w_lds = (long)s.Kg * 128;
    const int KS = s.C / 32, NR = KS > 2 ? KS : 2;
    double best = 1e300;
    bool found = false;
    for (int tw = 1; tw <= s.Q && tw <= BM; ++tw) {
        int th = BM / tw;
        if (th > s.P) th = s.P;
        if (th < 1) continue;
        const int ph = (th - 1) * s.stride + (s.R - 1) * s.dil + 1;
        const int pw = (tw - 1) * s.stride + (s.S - 1) * s.dil + 1;
        const long npix = (long)ph * pw;
        const long patch_loads = (npix + 15) / 16;
        const long slice_bytes = patch_loads * 1024;
        if (w_lds + NR * slice_bytes + kResWaves * kResStage > kResLdsLimit) continue;
        if (npix >= (1 << 20)) continue;                                  // fp32 reciprocal index arithmetic
        if ((long)th * s.Q * s.K * 4 >= (1L << 31)) continue;             // in-block output offsets are 32-bit
        const long tiles = (long)((s.P + th - 1) / th) * ((s.Q + tw - 1) / tw);
        const double cost = (double)tiles * ((double)BM * RS + 4.0 * (double)npix);
        if (cost < best) {
            best = cost;
            found = true;
            g->TH = th; g->TW = tw; g->PH = ph; g->PW = pw; g->npix = (int)npix;
            g->tiles_h = (s.P + th - 1) / th; g->tiles_w = (s.Q + tw - 1) / tw;
            g->KS = KS; g->NR = NR; g->slice_bytes = (int)slice_bytes; g->w_bytes = (int)w_lds;
            g->patch_loads = (int)patch_loads;
            g->inv_tw = 1.0f / (float)tw; g->inv_pw = 1.0f / (float)pw; g->inv_s = 1.0f / (float)s.S;
        }
    }
    if (!found) return false;
    const long total = (long)s.N * g->tiles_h * g->tiles_w;
    if (total > 0x7fffffffL || RS * 4 * 1024L * KS != w_lds) return false;
    g->total_tiles = (int)total;
    if (cost_out) *cost_out = best * (double)s.N;
    return true;
}

template <typename T, typename TO, int MF>
hipError_t launch_res_t(const void* x, const void* w, void* y, const ConvShape& s, ResGeom g, hipStream_t st) {
    const int lds_bytes = g.w_bytes + g.NR * g.slice_bytes + kResWaves * kResStage;
    auto kern = ires_kernel<T, TO, MF>;
    const int threads = (kResWaves + kResLoaders) * 64;
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, kResLdsLimit);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
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
    const int cap = g_max_workgroups.load(std::memory_order_relaxed);
    const long slots = cap > 0 ? cap : (long)device_cus() * occ;
    const long per = (g.total_tiles + slots - 1) / slots;
    const int nwg = (int)((g.total_tiles + per - 1) / per);
    g.tiles_base = g.total_tiles / nwg;
    g.tiles_rem = g.total_tiles % nwg;
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(threads), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y, s, g);
    return hipGetLastError();
}

template <int MF>
hipError_t launch_res_mf(const void* x, const void* w, void* y, const ConvShape& s, const ResGeom& g, int in_t, int out_t,
                         hipStream_t st) {
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_res_t<bf16_t, float, MF>(x, w, y, s, g, st);
        return launch_res_t<bf16_t, bf16_t, MF>(x, w, y, s, g, st);
    }
    if (out_t == OUT_F32) return launch_res_t<f16_t, float, MF>(x, w, y, s, g, st);
    return launch_res_t<f16_t, f16_t, MF>(x, w, y, s, g, st);
}

constexpr int kResMF[] = {7, 8};
const char* const kResNames[] = {"r448x64_f7_4+2", "r512x64_f8_4+2"};

}  // namespace

int resident_num_variants() { return 2; }
const char* resident_variant_name(int v) { return kResNames[v]; }

bool resident_supported(const ConvShape& s, int v) {
    ResGeom g;
    return v >= 0 && v < 2 && plan_res(s, kResMF[v], &g, nullptr);
}

// The variant with the lower modelled cost, or -1 when the layer does not fit the kernel.
int resident_choose(const ConvShape& s) {
    ResGeom g;
    double c7 = 0, c8 = 0;
    const bool ok7 = plan_res(s, 7, &g, &c7), ok8 = plan_res(s, 8, &g, &c8);
    if (!ok7 && !ok8) return -1;
    if (ok7 && ok8) return c7 <= c8 ? 0 : 1;
    return ok7 ? 0 : 1;
}

hipError_t launch_resident(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v,
                           hipStream_t st) {
    ResGeom g;
    if (v < 0 || v >= 2 || !plan_res(s, kResMF[v], &g, nullptr)) return hipErrorInvalidConfiguration;
    if (v == 0) return launch_res_mf<7>(x, w, y, s, g, in_t, out_t, st);
    return launch_res_mf<8>(x, w, y, s, g, in_t, out_t, st);
}

}  // namespace iconv

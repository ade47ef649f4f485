// Implicit channel-first im2col convolution as a blocked MFMA GEMM (paper section 5,
// "Block-level Channel-First im2col"): the equivalent GEMM  y[M x K] = A[M x Kg] * B[K x Kg]^T
// is tiled first, one workgroup per BM x BN output tile (no atomics), and inside a tile the
// K loop walks the decomposed 1x1 filters of section 3.2: tap (r, s) outer, channel chunk
// inner.  For one K step every A-tile row is one contiguous channel run of one input pixel
// (NHWC), so the lowered matrix is produced by address arithmetic alone and only ever exists
// as a BM x BK tile in LDS.
#include <atomic>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

// ---------------------------------------------------------------------------------------------
// Per-tap kernel: global memory -> LDS directly (buffer_load ... lds, 16 bytes per lane),
// ST stages deep, one barrier per K step.  One such instruction fills 1 KiB of LDS in lane
// order, so the chunk swizzle is applied on the global side: the lane that owns LDS slot
// (row, physical chunk) fetches logical chunk  physical ^ f(row).
//
// The loads are emitted as inline assembly on purpose: the compiler then does not pair every
// later LDS read with a wait for *all* outstanding loads, and the kernel places its own
// s_waitcnt vmcnt(n) so that the loads of the next ST-2 steps stay in flight during a step.
//
// PF = 1: the operand fragments of step i + 1 are read from LDS between the MFMAs of step i, and
// the fragment registers act as one more stage.  The epilogue goes through wave-private LDS
// staging areas (the stages are free by then), so that every store covers whole 128-byte lines.
// ---------------------------------------------------------------------------------------------
template <int V> struct StepTag { static constexpr int value = V; };

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int ST, int PF>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
igemm_dma_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s,
                 const int tiles_n, const int xcd_aware) {
    constexpr int WAVES_N = BN / WN;
    constexpr int WAVES = (BM / WM) * WAVES_N;
    constexpr int CPR = BK / 8;                 // 16-byte chunks per tile row
    constexpr int RPB = 64 / CPR;               // tile rows one wave-wide load covers
    constexpr int A_IT = BM / RPB / WAVES, B_IT = BN / RPB / WAVES;   // loads per wave per step
    constexpr int LPS = A_IT + B_IT;
    constexpr int MI = WM / 32, NI = WN / 32, KI = BK / 16;
    constexpr int STAGE_CHUNKS = (BM + BN) * CPR;
    static_assert((BM / RPB) % WAVES == 0 && (BN / RPB) % WAVES == 0, "tile rows must divide over the waves");
    static_assert(ST >= 2 && LPS * (ST - 2) < 64, "too many loads in flight for vmcnt");
    typedef typename Elem<T>::frag frag_t;

    extern __shared__ u32x4 lds[];              // ST stages of [A: BM x CPR][B: BN x CPR] chunks

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform, lives in an SGPR
    const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
    const int tile = xcd_aware ? xcd_remap(blockIdx.x, gridDim.x) : (int)blockIdx.x;
    const int tile_n = tile % tiles_n, tile_m = tile / tiles_n;
    const int m0 = tile_m * BM, k0 = tile_n * BN;

    const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * s.C * (uint32_t)sizeof(T);
    const uint32_t w_bytes = (uint32_t)s.K * s.Kg * (uint32_t)sizeof(T);
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
    const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds;

    // ---- loader state.  Load j of this wave covers tile rows (wave + j*WAVES)*RPB .. +RPB; lane l
    // owns row +l/CPR, physical chunk l%CPR of it, and fetches the logical chunk that belongs there.
    const int lr = lane / CPR, pc = lane % CPR;
    uint32_t a_off[A_IT];
    int a_h0[A_IT], a_w0[A_IT], a_ch[A_IT];
#pragma unroll
    for (int j = 0; j < A_IT; ++j) {
        const int row = (wave + j * WAVES) * RPB + lr;
        const int m = m0 + row;
        a_ch[j] = swz<CPR>(row, pc) * 8;        // first channel (within the K step) this lane fetches
        if (m < s.M) {
            const int n = m / s.PQ;
            const int pq = m - n * s.PQ;
            const int p = pq / s.Q, q = pq - p * s.Q;
            a_h0[j] = p * s.stride - s.pad;
            a_w0[j] = q * s.stride - s.pad;
            a_off[j] = (uint32_t)(((n * s.H + a_h0[j]) * s.W + a_w0[j]) * s.C + a_ch[j]) * (uint32_t)sizeof(T);
        } else {
            a_h0[j] = -(1 << 28);               // never in bounds
            a_w0[j] = 0;
            a_off[j] = 0;
        }
    }
    uint32_t b_off[B_IT];
    int b_ch[B_IT];
#pragma unroll
    for (int j = 0; j < B_IT; ++j) {
        const int row = (wave + j * WAVES) * RPB + lr;
        const int kf = k0 + row;
        b_ch[j] = swz<CPR>(row, pc) * 8;
        b_off[j] = kf < s.K ? (uint32_t)(kf * s.Kg + b_ch[j]) * (uint32_t)sizeof(T) : w_bytes;
    }

    int r = 0, ss = 0, c0 = 0;                  // K-step state of the loader (wave-uniform)
    const int steps = s.R * s.S * ((s.C + BK - 1) / BK);

    // Issues the LPS loads of the loader's current K step into `stage`, then advances the step.
    // Past the last step every lane's offset is out of range: the loads still count in vmcnt
    // (which keeps the wait arithmetic uniform) but fetch nothing.
    auto issue = [&](int stage, bool live) {
        const int dh = r * s.dil, dw = ss * s.dil;
        const uint32_t a_delta = (uint32_t)((dh * s.W + dw) * s.C + c0) * (uint32_t)sizeof(T);
        const uint32_t b_delta = (uint32_t)((r * s.S + ss) * s.C + c0) * (uint32_t)sizeof(T);
        const uint32_t stage_addr = lds_base + (uint32_t)stage * (STAGE_CHUNKS * 16);
#pragma unroll
        for (int j = 0; j < A_IT; ++j) {
            const bool ok = live && (c0 + a_ch[j]) < s.C && (unsigned)(a_h0[j] + dh) < (unsigned)s.H &&
                            (unsigned)(a_w0[j] + dw) < (unsigned)s.W;
            dma16(x_rsrc, ok ? a_off[j] + a_delta : x_bytes, stage_addr + (uint32_t)((wave + j * WAVES) * 1024));
        }
#pragma unroll
        for (int j = 0; j < B_IT; ++j) {
            const bool ok = live && (c0 + b_ch[j]) < s.C && b_off[j] != w_bytes;
            dma16(w_rsrc, ok ? b_off[j] + b_delta : w_bytes,
                  stage_addr + (uint32_t)(BM * CPR * 16 + (wave + j * WAVES) * 1024));
        }
        c0 += BK;
        if (c0 >= s.C) {
            c0 = 0;
            if (++ss == s.S) { ss = 0; ++r; }
        }
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    const int frow = lane & 31, fk = lane >> 5;

    if constexpr (PF != 0) {
        // ---- prefetching pipeline: the operand fragments of step i + 1 are read from LDS between the
        // MFMAs of step i (a wave issues in order, so only what sits between its MFMAs runs in
        // their shadow), and the global loads of a later step follow the MFMAs.  The fragment
        // registers act as one more stage: the ring holds ST stages in flight or landed, stage
        // i + 1 must have landed at the barrier of step i, and the slot of stage i is refilled right
        // after that barrier (every wave read it during step i - 1).
        int a_idx[MI][KI], b_idx[NI][KI];       // fragment positions within a stage (16-byte units)
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = wave_m * WM + mi * 32 + frow;
#pragma unroll
            for (int kk = 0; kk < KI; ++kk) a_idx[mi][kk] = row * CPR + swz<CPR>(row, kk * 2 + fk);
        }
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int row = wave_n * WN + ni * 32 + frow;
#pragma unroll
            for (int kk = 0; kk < KI; ++kk) b_idx[ni][kk] = BM * CPR + row * CPR + swz<CPR>(row, kk * 2 + fk);
        }
        frag_t af[2][KI][MI], bfr[2][KI][NI];
        auto read_stage = [&](int stage, auto BUF) __attribute__((always_inline)) {
            constexpr int buf = decltype(BUF)::value;
            const u32x4* S = lds + stage * STAGE_CHUNKS;
#pragma unroll
            for (int kk = 0; kk < KI; ++kk) {
#pragma unroll
                for (int mi = 0; mi < MI; ++mi) af[buf][kk][mi] = __builtin_bit_cast(frag_t, S[a_idx[mi][kk]]);
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) bfr[buf][kk][ni] = __builtin_bit_cast(frag_t, S[b_idx[ni][kk]]);
            }
        };
#pragma unroll
        for (int j = 0; j < ST; ++j) issue(j, j < steps);
        wait_vmcnt<LPS * (ST - 1)>();           // stage 0
        __syncthreads();
        read_stage(0, StepTag<0>{});
        int nxt = 1;                            // ring slot of the step after the current one
        auto one_step = [&](int step, auto PAR) __attribute__((always_inline)) {
            constexpr int cur = decltype(PAR)::value;
            wait_vmcnt<LPS * (ST - 2)>();       // this wave's loads of step + 1 have landed
            __syncthreads();                    // ... everyone's have, and nobody reads the slot of `step` any more
            // The slot of `step` is refilled by half of the waves before their MFMAs and by the other half after
            // theirs: a wave is held while it issues its loads, and the two waves of a SIMD (w and w + WAVES / 2)
            // then take turns at the matrix pipe instead of both issuing loads at the same time.
            const bool early = WAVES >= 8 && wave < WAVES / 2;
            if (early) {
                issue(nxt == 0 ? ST - 1 : nxt - 1, step + ST < steps);
                __builtin_amdgcn_sched_barrier(0);
            }
            read_stage(nxt, StepTag<cur ^ 1>{});
#pragma unroll
            for (int kk = 0; kk < KI; ++kk)
#pragma unroll
                for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                    for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Elem<T>::mfma32(bfr[cur][kk][ni], af[cur][kk][mi], acc[mi][ni]);
            constexpr int NM = KI * MI * NI, NR = KI * (MI + NI), RPM = (NR + NM - 1) / NM;
#pragma unroll
            for (int i = 0; i < NM; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);      // MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 2, 0);      // address arithmetic of the reads (measured: -1 % against none, 1 or 4)
                __builtin_amdgcn_sched_group_barrier(0x100, RPM, 0);    // LDS reads of the next step
            }
            __builtin_amdgcn_sched_barrier(0);
            if (!early) issue(nxt == 0 ? ST - 1 : nxt - 1, step + ST < steps);     // refill the slot of `step`
            nxt = nxt + 1 == ST ? 0 : nxt + 1;
        };
        for (int step = 0; step < steps;) {
            one_step(step, StepTag<0>{});
            if (++step < steps) {
                one_step(step, StepTag<1>{});
                ++step;
            }
        }
    } else {
#pragma unroll
    for (int j = 0; j < ST - 1; ++j) issue(j, j < steps);

    int stage = 0, fill = ST - 1;               // stage being consumed / stage being refilled
    for (int step = 0; step < steps; ++step) {
        wait_vmcnt<LPS * (ST - 2)>();           // this wave's loads of `step` have landed
        __syncthreads();                        // ... everyone's have, and the stage consumed last step is free
        // all operand fragments of the step first, then (while they are in flight) the global
        // loads of a later step, then the MFMAs
        const u32x4* A = lds + stage * STAGE_CHUNKS;
        const u32x4* Bt = A + BM * CPR;
        frag_t af[KI][MI], bfr[KI][NI];
#pragma unroll
        for (int mi = 0; mi < MI; ++mi) {
            const int row = wave_m * WM + mi * 32 + frow;
#pragma unroll
            for (int kk = 0; kk < KI; ++kk) af[kk][mi] = __builtin_bit_cast(frag_t, A[row * CPR + swz<CPR>(row, kk * 2 + fk)]);
        }
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int row = wave_n * WN + ni * 32 + frow;
#pragma unroll
            for (int kk = 0; kk < KI; ++kk) bfr[kk][ni] = __builtin_bit_cast(frag_t, Bt[row * CPR + swz<CPR>(row, kk * 2 + fk)]);
        }
        __builtin_amdgcn_sched_barrier(0);
        issue(fill, step + ST - 1 < steps);
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int kk = 0; kk < KI; ++kk)
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Elem<T>::mfma32(bfr[kk][ni], af[kk][mi], acc[mi][ni]);
        stage = stage + 1 == ST ? 0 : stage + 1;
        fill = fill + 1 == ST ? 0 : fill + 1;
    }
    }
    wait_vmcnt<0>();                            // drain the trailing no-op loads before the wave ends

    // ---- epilogue through LDS (whole 128-byte lines per store) when y rows are made of 16-byte
    // pieces and the tile's offsets fit the 32-bit buffer offset; the stages are free once every
    // wave has left the K loop.
    if ((s.K & 3) == 0 && (long long)s.K * BM * (long long)sizeof(TO) < 0x7fffffffLL) {
        __syncthreads();
        char* stg = reinterpret_cast<char*>(lds) + wave * kFragStageBytes;
        static_assert(WAVES * kFragStageBytes <= ST * STAGE_CHUNKS * 16, "staging must fit the stages");
        const size_t org = (size_t)m0 * s.K;
        const size_t rem = ((size_t)s.M * s.K - org) * sizeof(TO);
        // at most 2^31 - 1 bytes in range, so that the drop marker below stays out of range
        const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + org, 0, rem > 0x7fffffffull ? 0x7fffffffu : (uint32_t)rem,
                                                               kRsrcFlags);
        const int rows_left = s.M - m0;         // rows of this tile that exist
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int col0 = k0 + wave_n * WN + ni * 32;
                const int row0 = wave_m * WM + mi * 32;
                const bool pieces_ok = col0 + 4 * (lane & 7) + 3 < s.K;
                store_frag_staged<TO>(stg, acc[mi][ni], lane, y_rsrc, pieces_ok, [&](int i) {
                    const int row = row0 + i;
                    return row < rows_left ? (uint32_t)(row * s.K + col0) * (uint32_t)sizeof(TO) : 0x80000000u;
                });
            }
        return;
    }

    // ---- epilogue.  The filter fragment is the MFMA's row operand and the pixel fragment its
    // column operand, so lane l holds output row (pixel) l%32 of the 32-row block and, in
    // accumulator element v, filter 8*(v/4) + 4*(l/32) + v%4 of the 32-wide block: four
    // consecutive filters per group of four elements, stored as one 16-byte (fp32) or 8-byte
    // (16-bit) piece of the pixel's y row.
    const bool vec_ok = (s.K & 3) == 0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int row = m0 + wave_m * WM + mi * 32 + frow;
        if (row < s.M) {
            TO* yrow = y + (size_t)row * s.K;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int col = k0 + wave_n * WN + ni * 32 + 8 * gq + 4 * fk;
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

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int ST, int PF = 0>
hipError_t launch_dma(const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    constexpr int THREADS = (BM / WM) * (BN / WN) * 64;
    constexpr int LDS_BYTES = ST * (BM + BN) * BK * 2;
    static_assert(LDS_BYTES <= 160 * 1024, "stages do not fit the 160 KiB LDS");
    const int tiles_m = (s.M + BM - 1) / BM, tiles_n = (s.K + BN - 1) / BN;
    auto kern = igemm_dma_kernel<T, TO, BM, BN, BK, WM, WN, ST, PF>;
    if (LDS_BYTES > 64 * 1024) {
        // once per kernel and process; a failed attempt is retried by the next call
        static std::atomic<bool> raised{false};
        if (!raised.load(std::memory_order_acquire)) {
            hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, LDS_BYTES);
            if (e != hipSuccess) return e;
            raised.store(true, std::memory_order_release);
        }
    }
    hipLaunchKernelGGL(kern, dim3(tiles_m * tiles_n), dim3(THREADS), LDS_BYTES, st, (const T*)x, (const T*)w, (TO*)y, s,
                       tiles_n, 1);
    return hipGetLastError();
}

// Kernel table of this file (per-tap loader, direct-to-LDS, ST stages).  Name: BMxBNxBK, wave
// tile, stages.
#define ICONV_VARIANTS(X)                                                                \
    X(kD128x64, "d128x64x64_w64x32_s4", (launch_dma<T, TO, 128, 64, 64, 64, 32, 4>))          \
    X(kD256x128, "d256x128x64_w64x64_s3", (launch_dma<T, TO, 256, 128, 64, 64, 64, 3>))       \
    X(kD256x256, "d256x256x32_w128x64_s3", (launch_dma<T, TO, 256, 256, 32, 128, 64, 3>))     \
    X(kD64x64, "d64x64x64_w32x32_s4", (launch_dma<T, TO, 64, 64, 64, 32, 32, 4>))             \
    X(kD128x128, "d128x128x64_w64x32_s3", (launch_dma<T, TO, 128, 128, 64, 64, 32, 3>))       \
    X(kD128x128Pf, "d128x128x64_w64x32_s3_pf", (launch_dma<T, TO, 128, 128, 64, 64, 32, 3, 1>))

#define X_ENUM(i, name, fn) i,
enum DmaVariant { ICONV_VARIANTS(X_ENUM) kNumVariants };
#undef X_ENUM
#define X_NAME(i, name, fn) name,
const char* const kVariantNames[] = {ICONV_VARIANTS(X_NAME)};
#undef X_NAME
static_assert(sizeof(kVariantNames) / sizeof(kVariantNames[0]) == kNumVariants, "one name per kernel");

template <typename T, typename TO>
hipError_t launch_variant(int v, const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    switch (v) {
#define X_CASE(i, name, fn) \
    case i: return fn(x, w, y, s, st);
        ICONV_VARIANTS(X_CASE)
#undef X_CASE
        default: return hipErrorInvalidValue;
    }
}

// Default kernel choice.  Returns an index into the combined table (this file's kernels first,
// then the patch-reuse kernels).  Layers with more than one tap and stride 1 take a patch-reuse
// kernel (input traffic drops by about R*S); 1x1 layers have nothing to reuse, and for strided
// layers the patch holds (stride^2 - 1)/stride^2 pixels a tap never reads, so both stay with the
// per-tap loader.  Tile sizes follow the output size: big tiles when there are enough of them
// to fill 256 compute units, small ones otherwise.
int pointwise_index() { return kNumVariants + patch_num_variants() + resident_num_variants(); }

int choose_variant(const ConvShape& s) {
    const long tiles_256x128 = (long)((s.M + 255) / 256) * ((s.K + 127) / 128);
    const int P0 = kNumVariants;
    if (s.stride == 1) {
        // few channels and filters (1x1 layers included): filters and patch resident in LDS
        const int rv = resident_choose(s);
        if (rv >= 0) return P0 + patch_num_variants() + rv;
    }
    if (s.R * s.S > 1 && s.stride == 1) {
        int v;
        const long tiles_256x64 = (long)((s.M + 255) / 256) * ((s.K + 63) / 64);
        if (s.K <= 64)                                // p256x64 (eight compute waves of 32x64), p128x64 or p64x64
            v = (s.M + 255) / 256 >= 128 ? kP256x64 : (s.M + 127) / 128 >= 128 ? kP128x64 : kP64x64;
        else if (tiles_256x128 >= 190)                // p256x128; with many channel chunks per tap, operands prefetched
            v = s.C >= 256 ? kP256x128Pf : kP256x128; // one group of K slices ahead
        else if (tiles_256x64 >= 190) v = kP256x64;   // p256x64 when that still gives most compute units a tile
        else if (s.C % 128 == 0) {                    // p64x128 (many small tiles), 128-channel chunks: half the steps;
            v = kP64x128C128;                         // with one round of workgroups, two compute waves per tile
            const long tiles_64x128 = (long)((s.M + 63) / 64) * ((s.K + 127) / 128);   // position on half the K slices each
            if (tiles_64x128 <= device_cus() && patch_supported(s, kP64x128C128K2)) v = kP64x128C128K2;
        }
        else v = kP64x128Pf;                          // p64x128, prefetching
        if (patch_supported(s, v)) return P0 + v;
        if (v != kP64x128 && s.K > 64 && patch_supported(s, kP64x128)) return P0 + kP64x128;
    }
    if (s.R * s.S == 1) {
        const int pv = pointwise_choose(s);
        if (pv >= 0) return pointwise_index() + pv;
        const long tiles_256x256 = (long)((s.M + 255) / 256) * ((s.K + 255) / 256);
        if (s.K > 128 && tiles_256x256 >= 160) return kD256x256;
        if (tiles_256x128 >= 160) return kD256x128;
        if (s.K <= 64) return kD128x64;
        return (long)((s.M + 127) / 128) * ((s.K + 127) / 128) >= 160 ? kD128x128 : kD64x64;
    }
    if (s.K <= 64) return kD128x64;
    const long tiles_128x128 = (long)((s.M + 127) / 128) * ((s.K + 127) / 128);
    // d128x128x64 (operands prefetched a step ahead) while its tiles fit one round of workgroups; d256x128x64 when
    // they do not and the larger tiles still reach half the compute units; d64x64x64 for very small outputs
    if (tiles_128x128 > device_cus() && tiles_256x128 >= device_cus() / 2) return kD256x128;
    return tiles_128x128 >= 128 ? kD128x128Pf : kD64x64;
}

}  // namespace

// Variant numbering seen through the C ABI: the per-tap kernels of this file first, then the
// patch-reuse kernels, then the resident-filter kernels, then the pixel-resident 1x1 kernels.
int mfma_num_variants() { return pointwise_index() + pointwise_num_variants(); }
const char* mfma_variant_name(int v) {
    if (v < kNumVariants) return kVariantNames[v];
    if (v < kNumVariants + patch_num_variants()) return patch_variant_name(v - kNumVariants);
    if (v < pointwise_index()) return resident_variant_name(v - kNumVariants - patch_num_variants());
    return pointwise_variant_name(v - pointwise_index());
}

int mfma_default_variant(const ConvShape& s) { return choose_variant(s); }

bool mfma_variant_accepts(const ConvShape& s, int v) {
    const int R0 = kNumVariants + patch_num_variants();
    if (v < 0 || v >= mfma_num_variants()) return false;
    if (v >= pointwise_index()) return pointwise_supported(s);
    if (v >= R0) return resident_supported(s, v - R0);
    if (v >= kNumVariants) return patch_supported(s, v - kNumVariants);
    return true;
}

hipError_t launch_mfma(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int variant,
                       hipStream_t st) {
    const int R0 = kNumVariants + patch_num_variants();        // first resident-filter variant
    const int A0 = pointwise_index();
    if (variant >= A0 && variant < mfma_num_variants() && pointwise_supported(s)) return launch_pointwise(x, w, y, s, in_t, out_t, variant - A0, st);
    if (variant >= R0 && variant < A0 && resident_supported(s, variant - R0))
        return launch_resident(x, w, y, s, in_t, out_t, variant - R0, st);
    if (variant >= kNumVariants && variant < R0 && patch_supported(s, variant - kNumVariants))
        return launch_patch(x, w, y, s, in_t, out_t, variant - kNumVariants, st);
    int v = variant;
    if (v < 0 || v >= kNumVariants) v = choose_variant(s);    // also when a forced kernel does not fit the layer
    if (v >= A0) return launch_pointwise(x, w, y, s, in_t, out_t, v - A0, st);
    if (v >= R0) return launch_resident(x, w, y, s, in_t, out_t, v - R0, st);
    if (v >= kNumVariants) return launch_patch(x, w, y, s, in_t, out_t, v - kNumVariants, st);
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_variant<bf16_t, float>(v, x, w, y, s, st);
        return launch_variant<bf16_t, bf16_t>(v, x, w, y, s, st);
    }
    if (out_t == OUT_F32) return launch_variant<f16_t, float>(v, x, w, y, s, st);
    return launch_variant<f16_t, f16_t>(v, x, w, y, s, st);
}

}  // namespace iconv

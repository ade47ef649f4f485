// Implicit channel-first im2col convolution as a blocked MFMA GEMM (paper section 5,
// "Block-level Channel-First im2col"): the equivalent GEMM  y[M x K] = A[M x Kg] * B[K x Kg]^T
// is tiled first, one workgroup per BM x BN output tile (no atomics), and inside a tile the
// K loop walks the decomposed 1x1 filters of section 3.2: tap (r, s) outer, channel chunk
// inner.  For one K step every A-tile row is one contiguous channel run of one input pixel
// (NHWC), so the lowered matrix is produced by address arithmetic alone and only ever exists
// as a BM x BK tile in LDS.
#include <atomic>

#include "iconv_common.h"

namespace iconv {

namespace {

// 16-byte-chunk swizzle of a tile row: keeps both the row-contiguous ds_write_b128 of the
// loader and the column-of-rows ds_read_b128 of the MFMA operand fetch spread over all banks.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;
// dword 3 of a raw buffer descriptor on gfx9: 32-bit data format, no swizzle, offsets checked
// against num_records in bytes
constexpr int kRsrcFlags = 0x00020000;

template <int CPR> __device__ __forceinline__ int swz(int row, int chunk) {
    constexpr int RP = (8 / CPR) > 0 ? (8 / CPR) : 1;  // tile rows per 128 bytes
    return chunk ^ (((row / RP) ^ (row >> 3)) & (CPR - 1));
}

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN>
__global__ void __launch_bounds__((BM / WM) * (BN / WN) * 64)
igemm_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const int tiles_n) {
    constexpr int WAVES_N = BN / WN;
    constexpr int THREADS = (BM / WM) * WAVES_N * 64;
    constexpr int CPR = BK / 8;                 // 16-byte chunks per tile row
    constexpr int ROWS_PER_PASS = THREADS / CPR;
    constexpr int A_IT = BM / ROWS_PER_PASS, B_IT = BN / ROWS_PER_PASS;
    constexpr int MI = WM / 32, NI = WN / 32, KI = BK / 16;
    static_assert(BM % ROWS_PER_PASS == 0 && BN % ROWS_PER_PASS == 0, "tile rows must divide over the loader");
    static_assert(A_IT >= 1 && B_IT >= 1, "tile too small for the workgroup");
    typedef typename Elem<T>::frag frag_t;

    __shared__ u32x4 lds[2][(BM + BN) * CPR];

    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave / WAVES_N, wave_n = wave % WAVES_N;
    const int tile_n = blockIdx.x % tiles_n, tile_m = blockIdx.x / tiles_n;
    const int m0 = tile_m * BM, k0 = tile_n * BN;

    // ---- per-thread loader state: which tile rows / chunk this thread fetches ----------------
    // All offsets are byte offsets into x / w, kept as wrapping 32-bit values (tensors are below
    // 2^31 elements, so a valid offset always fits).  Loads go through raw buffer descriptors:
    // an out-of-range offset returns zeros, which is how padded taps, rows past M, filters past
    // K and channel chunks past C are blanked without a branch.
    const int ch = tid % CPR;          // 16-byte chunk within a row (same for all passes)
    const int lrow = tid / CPR;        // first row
    const uint32_t x_bytes = (uint32_t)s.N * s.H * s.W * s.C * (uint32_t)sizeof(T);
    const uint32_t w_bytes = (uint32_t)s.K * s.Kg * (uint32_t)sizeof(T);
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), 0, x_bytes, kRsrcFlags);
    const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);
    uint32_t a_off[A_IT];
    int a_h0[A_IT], a_w0[A_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int m = m0 + lrow + i * ROWS_PER_PASS;
        if (m < s.M) {
            const int n = m / s.PQ;
            const int pq = m - n * s.PQ;
            const int p = pq / s.Q, q = pq - p * s.Q;
            a_h0[i] = p * s.stride - s.pad;
            a_w0[i] = q * s.stride - s.pad;
            a_off[i] = (uint32_t)(((n * s.H + a_h0[i]) * s.W + a_w0[i]) * s.C + ch * 8) * (uint32_t)sizeof(T);
        } else {
            a_h0[i] = -(1 << 28);      // never in bounds
            a_w0[i] = 0;
            a_off[i] = 0;
        }
    }
    uint32_t b_off[B_IT];
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int kf = k0 + lrow + i * ROWS_PER_PASS;
        b_off[i] = kf < s.K ? (uint32_t)(kf * s.Kg + ch * 8) * (uint32_t)sizeof(T) : w_bytes;  // past K: out of range
    }

    // K-step state (wave-uniform): tap (r, s) and channel chunk c0
    int r = 0, ss = 0, c0 = 0;
    const int steps = s.R * s.S * ((s.C + BK - 1) / BK);

    u32x4 a_reg[A_IT], b_reg[B_IT];

    auto fetch = [&]() {
        const int dh = r * s.dil, dw = ss * s.dil;
        const bool c_ok = (c0 + ch * 8) < s.C;
        const uint32_t a_delta = (uint32_t)((dh * s.W + dw) * s.C + c0) * (uint32_t)sizeof(T);
        const uint32_t b_delta = (uint32_t)((r * s.S + ss) * s.C + c0) * (uint32_t)sizeof(T);
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const bool ok = c_ok && (unsigned)(a_h0[i] + dh) < (unsigned)s.H && (unsigned)(a_w0[i] + dw) < (unsigned)s.W;
            a_reg[i] = __builtin_amdgcn_raw_buffer_load_b128(x_rsrc, (int)(ok ? a_off[i] + a_delta : x_bytes), 0, 0);
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const bool ok = c_ok && b_off[i] != w_bytes;
            b_reg[i] = __builtin_amdgcn_raw_buffer_load_b128(w_rsrc, (int)(ok ? b_off[i] + b_delta : w_bytes), 0, 0);
        }
        // advance to the next step: channel chunk fastest, then tap column, then tap row
        c0 += BK;
        if (c0 >= s.C) {
            c0 = 0;
            if (++ss == s.S) { ss = 0; ++r; }
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int row = lrow + i * ROWS_PER_PASS;
            lds[buf][row * CPR + swz<CPR>(row, ch)] = a_reg[i];
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int row = lrow + i * ROWS_PER_PASS;
            lds[buf][BM * CPR + row * CPR + swz<CPR>(row, ch)] = b_reg[i];
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

    fetch();
    stash(0);
    __syncthreads();

    for (int step = 0; step < steps; ++step) {
        const int buf = step & 1;
        const bool more = step + 1 < steps;
        if (more) fetch();
#pragma unroll
        for (int kk = 0; kk < KI; ++kk) {
            frag_t af[MI], bfr[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int row = wave_m * WM + mi * 32 + frow;
                af[mi] = __builtin_bit_cast(frag_t, lds[buf][row * CPR + swz<CPR>(row, kk * 2 + fk)]);
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int row = wave_n * WN + ni * 32 + frow;
                bfr[ni] = __builtin_bit_cast(frag_t, lds[buf][BM * CPR + row * CPR + swz<CPR>(row, kk * 2 + fk)]);
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Elem<T>::mfma32(af[mi], bfr[ni], acc[mi][ni]);
        }
        if (more) stash(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulators -> y (row-major M x K).  In a 32x32 accumulator block lane l
    // holds column l%32 and rows 8*(v/4) + 4*(l/32) + v%4, so each store covers 128-byte runs.
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int col = k0 + wave_n * WN + ni * 32 + frow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wave_m * WM + mi * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                if (row < s.M && col < s.K) y[(size_t)row * s.K + col] = to_out<TO>(acc[mi][ni][v]);
            }
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Pipelined kernel: global memory -> LDS directly (buffer_load ... lds, 16 bytes per lane),
// ST stages deep, one barrier per K step.  One such instruction fills 1 KiB of LDS in lane
// order, so the chunk swizzle is applied on the global side: the lane that owns LDS slot
// (row, physical chunk) fetches logical chunk  physical ^ f(row).
//
// The loads are emitted as inline assembly on purpose: the compiler then does not pair every
// later LDS read with a wait for *all* outstanding loads, and the kernel places its own
// s_waitcnt vmcnt(n) so that the loads of the next ST-2 steps stay in flight during a step.
// ---------------------------------------------------------------------------------------------
__device__ __forceinline__ void dma16(rsrc_t rsrc, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

// s_waitcnt vmcnt(n) with the other counters left alone (gfx9 encoding)
template <int N> __device__ __forceinline__ void wait_vmcnt() {
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// Workgroup id -> logical tile id such that the workgroups one XCD receives (ids congruent
// modulo 8, in dispatch order) cover one contiguous range of tiles: neighbouring tiles share
// input halo rows and filter tiles in that XCD's L2.
__device__ __forceinline__ int xcd_remap(int wg, int nwg) {
    const int per = nwg >> 3, rem = nwg & 7;
    const int xcd = wg & 7, j = wg >> 3;
    return xcd < rem ? xcd * (per + 1) + j : rem * (per + 1) + (xcd - rem) * per + j;
}

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int ST>
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

#pragma unroll
    for (int j = 0; j < ST - 1; ++j) issue(j, j < steps);

    int stage = 0, fill = ST - 1;               // stage being consumed / stage being refilled
    for (int step = 0; step < steps; ++step) {
        wait_vmcnt<LPS * (ST - 2)>();           // this wave's loads of `step` have landed
        __syncthreads();                        // ... everyone's have, and the stage consumed last step is free
        issue(fill, step + ST - 1 < steps);
        const u32x4* A = lds + stage * STAGE_CHUNKS;
        const u32x4* Bt = A + BM * CPR;
#pragma unroll
        for (int kk = 0; kk < KI; ++kk) {
            frag_t af[MI], bfr[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int row = wave_m * WM + mi * 32 + frow;
                af[mi] = __builtin_bit_cast(frag_t, A[row * CPR + swz<CPR>(row, kk * 2 + fk)]);
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int row = wave_n * WN + ni * 32 + frow;
                bfr[ni] = __builtin_bit_cast(frag_t, Bt[row * CPR + swz<CPR>(row, kk * 2 + fk)]);
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Elem<T>::mfma32(af[mi], bfr[ni], acc[mi][ni]);
        }
        stage = stage + 1 == ST ? 0 : stage + 1;
        fill = fill + 1 == ST ? 0 : fill + 1;
    }
    wait_vmcnt<0>();                            // drain the trailing no-op loads before the wave ends

#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
#pragma unroll
        for (int ni = 0; ni < NI; ++ni) {
            const int col = k0 + wave_n * WN + ni * 32 + frow;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wave_m * WM + mi * 32 + 8 * (v >> 2) + 4 * fk + (v & 3);
                if (row < s.M && col < s.K) y[(size_t)row * s.K + col] = to_out<TO>(acc[mi][ni][v]);
            }
        }
    }
}

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN>
hipError_t launch_one(const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    constexpr int THREADS = (BM / WM) * (BN / WN) * 64;
    const int tiles_m = (s.M + BM - 1) / BM, tiles_n = (s.K + BN - 1) / BN;
    hipLaunchKernelGGL((igemm_kernel<T, TO, BM, BN, BK, WM, WN>), dim3(tiles_m * tiles_n), dim3(THREADS), 0, st,
                       (const T*)x, (const T*)w, (TO*)y, s, tiles_n);
    return hipGetLastError();
}

template <typename T, typename TO, int BM, int BN, int BK, int WM, int WN, int ST>
hipError_t launch_dma(const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    constexpr int THREADS = (BM / WM) * (BN / WN) * 64;
    constexpr int LDS_BYTES = ST * (BM + BN) * BK * 2;
    static_assert(LDS_BYTES <= 160 * 1024, "stages do not fit the 160 KiB LDS");
    const int tiles_m = (s.M + BM - 1) / BM, tiles_n = (s.K + BN - 1) / BN;
    auto kern = igemm_dma_kernel<T, TO, BM, BN, BK, WM, WN, ST>;
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

// Kernel table.  r* = register-staged loader (two LDS buffers); d* = direct-to-LDS loader with
// the given number of stages.  Name: BMxBNxBK, wave tile, stages.
#define ICONV_VARIANTS(X)                      \
    X(0, "r128x128x32_w64x64", (launch_one<T, TO, 128, 128, 32, 64, 64>))      \
    X(1, "r128x64x32_w64x32", (launch_one<T, TO, 128, 64, 32, 64, 32>))        \
    X(2, "r128x128x64_w64x64", (launch_one<T, TO, 128, 128, 64, 64, 64>))      \
    X(3, "r64x64x64_w32x32", (launch_one<T, TO, 64, 64, 64, 32, 32>))          \
    X(4, "d128x128x32_w64x64_s3", (launch_dma<T, TO, 128, 128, 32, 64, 64, 3>)) \
    X(5, "d128x128x64_w64x64_s3", (launch_dma<T, TO, 128, 128, 64, 64, 64, 3>)) \
    X(6, "d128x128x64_w64x64_s4", (launch_dma<T, TO, 128, 128, 64, 64, 64, 4>)) \
    X(7, "d128x64x64_w64x32_s4", (launch_dma<T, TO, 128, 64, 64, 64, 32, 4>))   \
    X(8, "d256x64x64_w64x64_s3", (launch_dma<T, TO, 256, 64, 64, 64, 64, 3>))   \
    X(9, "d256x128x64_w128x64_s3", (launch_dma<T, TO, 256, 128, 64, 128, 64, 3>)) \
    X(10, "d256x128x64_w64x64_s3", (launch_dma<T, TO, 256, 128, 64, 64, 64, 3>))  \
    X(11, "d256x128x32_w64x64_s4", (launch_dma<T, TO, 256, 128, 32, 64, 64, 4>))  \
    X(12, "d256x256x32_w128x64_s3", (launch_dma<T, TO, 256, 256, 32, 128, 64, 3>)) \
    X(13, "d256x256x64_w128x64_s2", (launch_dma<T, TO, 256, 256, 64, 128, 64, 2>)) \
    X(14, "d64x64x64_w32x32_s4", (launch_dma<T, TO, 64, 64, 64, 32, 32, 4>))       \
    X(15, "d64x128x64_w32x64_s4", (launch_dma<T, TO, 64, 128, 64, 32, 64, 4>))     \
    X(16, "d128x128x64_w64x32_s3", (launch_dma<T, TO, 128, 128, 64, 64, 32, 3>))

#define X_NAME(i, name, fn) name,
const char* const kVariantNames[] = {ICONV_VARIANTS(X_NAME)};
#undef X_NAME
constexpr int kNumVariants = sizeof(kVariantNames) / sizeof(kVariantNames[0]);

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

// Default tile choice: narrow N tile for layers with few filters, small tiles when the output
// has too few rows to give every compute unit a 128-row tile.
int choose_variant(const ConvShape& s) {
    const long tiles128 = (long)((s.M + 127) / 128) * ((s.K + 127) / 128);
    if (s.K <= 64) return 1;
    if (tiles128 < 256) return 3;
    return 0;
}

}  // namespace

int mfma_num_variants() { return kNumVariants; }
const char* mfma_variant_name(int v) { return kVariantNames[v]; }

hipError_t launch_mfma(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int variant,
                       hipStream_t st) {
    const int v = (variant >= 0 && variant < kNumVariants) ? variant : choose_variant(s);
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_variant<bf16_t, float>(v, x, w, y, s, st);
        return launch_variant<bf16_t, bf16_t>(v, x, w, y, s, st);
    }
    if (out_t == OUT_F32) return launch_variant<f16_t, float>(v, x, w, y, s, st);
    return launch_variant<f16_t, f16_t>(v, x, w, y, s, st);
}

}  // namespace iconv

// 1x1 convolutions (any stride): the pixel-resident kernel.
//
// A 1x1 layer is the GEMM  y[M x K] = x'[M x C] * w[K x C]^T  whose rows are the (sampled) input pixels
// themselves: the per-tap decomposition of the paper (section 3.2) with a single tap.  Its cost on
// this chip is the write of y, so the kernel is built around keeping the stores going:
//
//  * a workgroup owns up to 128 consecutive output pixels; their C channels are loaded into LDS once,
//    and every compute wave takes the fragments of its 32 pixels into registers for the whole kernel,
//    so a K step is one filter-fragment read and one MFMA;
//  * the filters stream through a ring of eight LDS slots in tiles of 32 (eight loader waves, global ->
//    LDS DMA), requested up to three pairs of tiles ahead of their use;
//  * two TEAMS of four compute waves each take one tile of a pair (four waves x 32 pixels x 32 filters),
//    multiply it and write it out through the staged stores; one workgroup barrier per pair hands the
//    slots back to the loader waves.  Eight waves with a tile each keep the matrix pipe and the store
//    path busier than one large tile per workgroup, and the next pairs land meanwhile.
//    (A form in which one team multiplies while the other stores, tile by tile, measured slower: the
//    two do not overlap well on one compute unit.)
//
// LDS: [pixels: 128 rows x 2C bytes][filters: 4 slots x 32 rows x 2C bytes][staging: 2 KiB per compute
// wave]; once the pixel fragments are in registers the pixel region serves as four more filter slots.
// Rows hold their 16-byte chunks XOR-swizzled so that the MFMA operand read (32 consecutive
// rows, one chunk per half-wave) is free of bank conflicts (swz<CPR>, the function of the other MFMA
// kernels).  The DMA fills write lane-linear and apply the swizzle on the global side.
#include <atomic>

#include "iconv_common.h"
#include "iconv_device.h"
#include "iconv_host.h"

namespace iconv {

namespace {

constexpr int kPwBM = 128;        // pixels per workgroup at most
constexpr int kPwBN = 32;         // filters per tile
constexpr int kPwSlots = 8;       // filter tiles in LDS: a pair in use, up to three pairs landing
constexpr int kPwWaves = 16;      // 2 teams x 4 compute waves + 8 loader waves
constexpr int kPwLoaders = 8;
constexpr int kPwStage = kFragStageBytes;
constexpr uint32_t kPwDrop = 0x80000000u;   // offset that every buffer of this kernel treats as out of range

struct PwGeom {
    int rows_per_wg;     // output pixels per workgroup (<= 128)
    int tiles_n;         // filter tiles of 32
    float inv_q, inv_p;  // 1 / Q, 1 / P
};

// Byte offset in LDS of filter-tile slot s (0..7).  Slots 0-3 follow the pixel region; slots 4-7 ARE the pixel
// region, which is free once every compute wave has taken its pixel fragments into registers.
template <int CPR> __device__ __forceinline__ uint32_t pw_slot(int s) {
    constexpr uint32_t A_BYTES = kPwBM * CPR * 16, B_BYTES = kPwBN * CPR * 16;
    static_assert(4 * B_BYTES <= A_BYTES, "four tiles fit the pixel region");
    return s < 4 ? A_BYTES + (uint32_t)s * B_BYTES : (uint32_t)(s - 4) * B_BYTES;
}

template <typename T, typename TO, int CPR>
__global__ void __launch_bounds__(kPwWaves * 64)
ipw_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const PwGeom g) {
    static_assert(CPR == 8 || CPR == 16 || CPR == 32, "64, 128 or 256 channels");
    typedef typename Elem<T>::frag frag_t;
    constexpr int PITCH = CPR * 16;             // bytes of an LDS row (all channels of a pixel or filter)
    constexpr int RPI = 64 / CPR;               // rows one wave-wide DMA instruction fills
    constexpr int NA = kPwBM / RPI;             // instructions for the pixel rows
    constexpr int NB = kPwBN / RPI;             // instructions for one filter tile
    constexpr int KK = CPR / 2;                 // K slices of 16 channels
    constexpr int A_BYTES = kPwBM * PITCH, B_BYTES = kPwBN * PITCH;
    constexpr int LPT = (NB + kPwLoaders - 1) / kPwLoaders;     // loads per loader wave and filter tile

    extern __shared__ u32x4 lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds;

    const int m0 = blockIdx.x * g.rows_per_wg;
    const int rows = min(g.rows_per_wg, s.M - m0);          // >= 1 by construction of the grid
    // first pixel of the workgroup, decoded once
    const int n0 = m0 / s.PQ;
    const int rem0 = m0 - n0 * s.PQ;
    const int p0 = rem0 / s.Q;
    const int q0 = rem0 - p0 * s.Q;

    // ---- buffers.  x is addressed from the start of image n0: the at most 128 pixels of the workgroup
    // lie in a few consecutive images, whose bytes the host has checked to stay below 2^31.
    const size_t x_off = (size_t)n0 * s.H * s.W * s.C;
    const size_t x_rem = ((size_t)s.N * s.H * s.W * s.C - x_off) * 2u;
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x) + x_off, 0, x_rem > kPwDrop ? kPwDrop : (uint32_t)x_rem,
                                                           kRsrcFlags);
    const uint32_t w_bytes = (uint32_t)s.K * s.C * 2u;      // < 2^31 (host)
    const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);

    const int r_in = lane / CPR, pc = lane % CPR;           // row within an instruction, physical chunk
    // global byte offset of the lane's chunk of pixel row `row` (0..127) of the workgroup, or kPwDrop
    auto a_offset = [&](int row) -> uint32_t {
        const int lc = swz<CPR>(row, pc);                // the swizzle is an involution on the chunk number
        const int qq = q0 + row;
        const int dp = (int)(((float)qq + 0.5f) * g.inv_q);     // exact: qq < Q + 128, Q < 2^14 (host)
        const int q = qq - dp * s.Q;
        const int pp = p0 + dp;
        const int dn = (int)(((float)pp + 0.5f) * g.inv_p);
        const int p = pp - dn * s.P;
        const int h = p * s.stride - s.pad, ww = q * s.stride - s.pad;
        const bool ok = row < rows && (unsigned)h < (unsigned)s.H && (unsigned)ww < (unsigned)s.W;
        return ok ? (uint32_t)(((dn * s.H + h) * s.W + ww) * s.C + lc * 8) * 2u : kPwDrop;
    };
    // global byte offset of the lane's chunk of filter row `row` (0..63) of filter tile `tile`
    auto b_offset = [&](int tile, int row) -> uint32_t {
        const int lc = swz<CPR>(row, pc);
        const int k = tile * kPwBN + row;
        return k < s.K ? (uint32_t)(k * s.C + lc * 8) * 2u : kPwDrop;
    };

    // ---- phase 0: the pixels and filter tiles 0 and 1, one share per wave (all sixteen issue)
#pragma unroll
    for (int i = 0; i < (NA + 2 * NB + kPwWaves - 1) / kPwWaves; ++i) {
        const int j = wave + i * kPwWaves;                  // uniform
        if (j < NA) {
            dma16(x_rsrc, a_offset(j * RPI + r_in), lds_base + (uint32_t)j * 1024u);
        } else if (j < NA + 2 * NB) {
            const int jb = j - NA;                          // tile jb / NB, instruction jb % NB of it
            dma16(w_rsrc, b_offset(jb / NB, (jb % NB) * RPI + r_in), lds_base + A_BYTES + (uint32_t)jb * 1024u);
        }
    }

    const int NT = g.tiles_n;
    const int NP = (NT + 1) / 2;                            // ticks: pairs of filter tiles
    if (wave >= 8) {
        // =========================== loader waves ===========================================
        const int lw = wave - 8;
        auto request = [&](int tile) {                      // this wave's loads of filter tile `tile`, if there is one
            if (tile >= NT) return;
            const uint32_t slot = lds_base + pw_slot<CPR>(tile & (kPwSlots - 1));
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int j = lw + i * kPwLoaders;          // uniform
                if (j < NB) dma16(w_rsrc, b_offset(tile, j * RPI + r_in), slot + (uint32_t)j * 1024u);
            }
        };
        // Loads complete in order within a wave: once at most the loads of the `after` tiles requested last are
        // outstanding, everything requested before them has landed.
        const bool issues = lw < NB;                        // with few loads per tile some loader waves have none
        auto landed_but = [&](int after) {
            if (!issues || after <= 0) wait_vmcnt<0>();
            else if (after == 1) wait_vmcnt<LPT>();
            else if (after == 2) wait_vmcnt<2 * LPT>();
            else if (after == 3) wait_vmcnt<3 * LPT>();
            else wait_vmcnt<4 * LPT>();
        };
        auto tiles_in = [&](int first, int last) { return max(0, min(NT - 1, last) - first + 1); };   // existing tiles of a range
        request(2);
        request(3);
        landed_but(tiles_in(2, 3));                         // phase 0 (pixels, tiles 0 and 1) is in LDS
        __syncthreads();
        for (int j = 0; j < NP; ++j) {
            // Tick j works on pair j (tiles 2j, 2j+1); pair j+1 must have landed when it ends.  Pairs up to j+3 may
            // be in flight: pair j+3 takes the slots of pair j-1, which every wave has left at the last barrier.
            // Nothing is requested in tick 0: pairs 2 and 3 go to the pixel region, which is read during tick 0.
            if (j == 1) {
                for (int t = 4; t < 10; ++t) request(t);
            } else if (j >= 2) {
                request(2 * j + 6);
                request(2 * j + 7);
            }
            landed_but(j == 0 ? 0 : tiles_in(2 * j + 4, 2 * j + 7));
            __syncthreads();
        }
        return;
    }

    // =========================== compute waves ==============================================
    const int team = wave >> 2;
    const int wq = wave & 3;                                // pixel quarter of the 128 x 32 tile
    const int frow = lane & 31, fk = lane >> 5;
    const char* lds_b = reinterpret_cast<const char*>(lds);
    const int arow = wq * 32 + frow;
    const uint32_t a_base = (uint32_t)(arow * PITCH + (swz<CPR>(arow, fk) << 4));
    const uint32_t b_base = (uint32_t)(frow * PITCH + (swz<CPR>(frow, fk) << 4));
    char* stg = reinterpret_cast<char*>(lds) + A_BYTES + 4 * B_BYTES + wave * kPwStage;
    const int c8 = lane & 7;

    // y is addressed from the workgroup's first pixel; 128 rows of K outputs stay below 2^31 bytes (host)
    const size_t y_off = (size_t)m0 * s.K;
    const size_t y_rem = ((size_t)s.M * s.K - y_off) * sizeof(TO);
    const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + y_off, 0, y_rem > kPwDrop ? kPwDrop : (uint32_t)y_rem, kRsrcFlags);

    floatx16 acc;
    // chunk 2*kk + fk of a row sits at (fk ^ swizzle) ^ 2*kk: the lane's address xor (kk << 5).
    // The wave's pixel fragments, all K slices, stay in registers from here on.
    frag_t areg[KK];
    auto read_pixels = [&]() {
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) areg[kk] = *reinterpret_cast<const frag_t*>(lds_b + (a_base ^ (uint32_t)(kk << 5)));
    };
    // Filter fragments are read two K slices ahead.
    auto multiply = [&](int slot) {
        const char* pb = lds_b + pw_slot<CPR>(slot);
        constexpr int AHEAD = 2;
        frag_t b[AHEAD];
#pragma unroll
        for (int kk = 0; kk < AHEAD; ++kk) b[kk] = *reinterpret_cast<const frag_t*>(pb + (b_base ^ (uint32_t)(kk << 5)));
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (kk == 0) {
                floatx16 z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0.f;
                acc = Elem<T>::mfma32(b[kk % AHEAD], areg[kk], z);
            } else {
                acc = Elem<T>::mfma32(b[kk % AHEAD], areg[kk], acc);
            }
            if (kk + AHEAD < KK)
                b[kk % AHEAD] = *reinterpret_cast<const frag_t*>(pb + (b_base ^ (uint32_t)((kk + AHEAD) << 5)));
        }
    };
    // The filters are the MFMA's row operand: lane l holds pixel l%32 of the fragment and, in accumulator
    // element v, filter 8*(v/4) + 4*(l/32) + v%4 of the tile's 32, which is what store_frag_staged expects.
    auto write_out = [&](int tile) {
        const int k_first = tile * kPwBN;
        const bool pieces_ok = k_first + 4 * c8 + 3 < s.K;
        const int r_first = wq * 32;
        store_frag_staged<TO>(stg, acc, lane, y_rsrc, pieces_ok, [&](int i) -> uint32_t {
            const int row = r_first + i;
            return row < rows ? (uint32_t)(row * s.K + k_first) * (uint32_t)sizeof(TO) : kPwDrop;
        });
    };

    wait_vmcnt<0>();
    __syncthreads();
    read_pixels();
    for (int j = 0; j < NP; ++j) {
        const int tile = 2 * j + team;
        if (tile < NT) {
            multiply(tile & (kPwSlots - 1));
            write_out(tile);
        }
        __syncthreads();
    }
}

// The same kernel with STORE WAVES: 2 teams x 4 compute waves, 4 loader waves and 4 store waves.  A wave that stores
// is held until the memory system has taken its data, and on this layer type the write of y is what takes
// longest, so here the compute waves never store: they deposit their fragments in one of two staging areas in
// LDS (each two tiles of 128 pixels x 32 filters in fp32, the layout of stage_off), and in the next tick the
// store waves carry that area out while the compute waves fill the other one.  One barrier per tick: it says
// that the tiles of the next pair have landed, that the staging area of this tick is complete and that the
// one of the last tick has been read.  The store waves finish with one more round after the last tick.
//
// LDS: [pixels][filter slots outside the pixel region][2 staging areas of 32 KiB].  The ring has eight slots
// (four pairs) up to 128 channels and six (three pairs) at 256, where four slots are the pixel region;
// the pixel region becomes slots once every compute wave has its pixel fragments in registers, which a
// barrier of its own announces.
constexpr int kPwsLoaders = 4;
constexpr int kPwsStaging = 2 * kPwBM * 128;      // bytes of one staging area: two tiles x 128 pixels x 32 fp32 outputs

template <int CPR> struct PwsLayout {
    static constexpr int SLOTS = CPR == 32 ? 6 : 8;
    static constexpr int OUTSIDE = SLOTS - 4;               // slots that are not the pixel region
    static constexpr int A_BYTES = kPwBM * CPR * 16, B_BYTES = kPwBN * CPR * 16;
    static constexpr int STG = A_BYTES + OUTSIDE * B_BYTES; // byte offset of the staging areas
    static constexpr int LDS_BYTES = STG + 2 * kPwsStaging;
    static_assert(4 * B_BYTES <= A_BYTES && LDS_BYTES <= 160 * 1024, "LDS of a compute unit");
    __device__ static uint32_t slot(int s) {
        return s < OUTSIDE ? (uint32_t)(A_BYTES + s * B_BYTES) : (uint32_t)((s - OUTSIDE) * B_BYTES);
    }
};

template <typename T, typename TO, int CPR>
__global__ void __launch_bounds__(kPwWaves * 64)
ipws_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const PwGeom g) {
    static_assert(CPR == 8 || CPR == 16 || CPR == 32, "64, 128 or 256 channels");
    typedef typename Elem<T>::frag frag_t;
    typedef PwsLayout<CPR> LY;
    constexpr int PITCH = CPR * 16;
    constexpr int RPI = 64 / CPR;
    constexpr int NA = kPwBM / RPI;
    constexpr int NB = kPwBN / RPI;
    constexpr int KK = CPR / 2;
    constexpr int A_BYTES = LY::A_BYTES;
    constexpr int LPT = (NB + kPwsLoaders - 1) / kPwsLoaders;
    constexpr int NPAIR = LY::SLOTS / 2;                    // pairs of tiles in the ring

    extern __shared__ u32x4 lds[];
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const uint32_t lds_base = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)lds;

    const int m0 = blockIdx.x * g.rows_per_wg;
    const int rows = min(g.rows_per_wg, s.M - m0);
    const int n0 = m0 / s.PQ;
    const int rem0 = m0 - n0 * s.PQ;
    const int p0 = rem0 / s.Q;
    const int q0 = rem0 - p0 * s.Q;

    const size_t x_off = (size_t)n0 * s.H * s.W * s.C;
    const size_t x_rem = ((size_t)s.N * s.H * s.W * s.C - x_off) * 2u;
    const rsrc_t x_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x) + x_off, 0, x_rem > kPwDrop ? kPwDrop : (uint32_t)x_rem,
                                                           kRsrcFlags);
    const uint32_t w_bytes = (uint32_t)s.K * s.C * 2u;
    const rsrc_t w_rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(w), 0, w_bytes, kRsrcFlags);

    const int r_in = lane / CPR, pc = lane % CPR;
    auto a_offset = [&](int row) -> uint32_t {
        const int lc = swz<CPR>(row, pc);
        const int qq = q0 + row;
        const int dp = (int)(((float)qq + 0.5f) * g.inv_q);
        const int q = qq - dp * s.Q;
        const int pp = p0 + dp;
        const int dn = (int)(((float)pp + 0.5f) * g.inv_p);
        const int p = pp - dn * s.P;
        const int h = p * s.stride - s.pad, ww = q * s.stride - s.pad;
        const bool ok = row < rows && (unsigned)h < (unsigned)s.H && (unsigned)ww < (unsigned)s.W;
        return ok ? (uint32_t)(((dn * s.H + h) * s.W + ww) * s.C + lc * 8) * 2u : kPwDrop;
    };
    auto b_offset = [&](int tile, int row) -> uint32_t {
        const int lc = swz<CPR>(row, pc);
        const int k = tile * kPwBN + row;
        return k < s.K ? (uint32_t)(k * s.C + lc * 8) * 2u : kPwDrop;
    };

    // ---- phase 0: the pixels and filter tiles 0 and 1 (slots 0 and 1), one share per wave (all sixteen issue)
#pragma unroll
    for (int i = 0; i < (NA + 2 * NB + kPwWaves - 1) / kPwWaves; ++i) {
        const int j = wave + i * kPwWaves;
        if (j < NA) {
            dma16(x_rsrc, a_offset(j * RPI + r_in), lds_base + (uint32_t)j * 1024u);
        } else if (j < NA + 2 * NB) {
            const int jb = j - NA;
            dma16(w_rsrc, b_offset(jb / NB, (jb % NB) * RPI + r_in), lds_base + A_BYTES + (uint32_t)jb * 1024u);
        }
    }

    const int NT = g.tiles_n;
    const int NP = (NT + 1) / 2;
    // Every role passes the same barriers: phase 0 landed, pixel fragments taken, then one per tick.
    if (wave >= 12) {
        // =========================== store waves ============================================
        // Store wave sw carries tile sw % 2 of the pair: the groups of eight pixels 2k + sw / 2, k = 0 .. 7 (with fewer
        // than 128 pixels in the workgroup the existing groups are then spread evenly over the four waves).
        const int sw = wave - 12;
        const int st = sw & 1, g0 = sw >> 1;
        const int l8 = lane >> 3, c8 = lane & 7;
        const size_t y_off = (size_t)m0 * s.K;
        const size_t y_rem = ((size_t)s.M * s.K - y_off) * sizeof(TO);
        const rsrc_t y_rsrc = __builtin_amdgcn_make_buffer_rsrc(y + y_off, 0, y_rem > kPwDrop ? kPwDrop : (uint32_t)y_rem, kRsrcFlags);
        const char* stg = reinterpret_cast<const char*>(lds) + LY::STG + st * (kPwsStaging / 2);
        uint32_t rd[8];
#pragma unroll
        for (int i = 0; i < 8; ++i) rd[i] = stage_off((2 * i + g0) * 8 + l8, c8);
        wait_vmcnt<0>();
        __syncthreads();
        __syncthreads();
        for (int j = 0; j <= NP; ++j) {
            if (j > 0) {                                    // the outputs of tick j - 1
                const char* area = stg + ((j - 1) & 1) * kPwsStaging;
                u32x4 v[8];
#pragma unroll
                for (int i = 0; i < 8; ++i) v[i] = *reinterpret_cast<const u32x4*>(area + rd[i]);
                const int tile = 2 * (j - 1) + st;
                const int k_first = tile * kPwBN;
                const bool pieces_ok = tile < NT && k_first + 4 * c8 + 3 < s.K;
#pragma unroll
                for (int i = 0; i < 8; ++i) {
                    const int row = (2 * i + g0) * 8 + l8;
                    if ((2 * i + g0) * 8 < rows) {          // uniform: some pixel of the instruction exists
                        const uint32_t ro = row < rows ? (uint32_t)(row * s.K + k_first + 4 * c8) * (uint32_t)sizeof(TO) : kPwDrop;
                        if (pieces_ok) store_piece<TO>(v[i], y_rsrc, ro);
                    }
                }
            }
            if (j < NP) __syncthreads();
        }
        return;
    }
    if (wave >= 8) {
        // =========================== loader waves ===========================================
        const int lw = wave - 8;
        auto request = [&](int tile) {
            if (tile >= NT) return;
            const uint32_t slot = lds_base + LY::slot(tile % LY::SLOTS);
#pragma unroll
            for (int i = 0; i < LPT; ++i) {
                const int j = lw + i * kPwsLoaders;
                if (j < NB) dma16(w_rsrc, b_offset(tile, j * RPI + r_in), slot + (uint32_t)j * 1024u);
            }
        };
        auto request_pair = [&](int p) {
            request(2 * p);
            request(2 * p + 1);
        };
        const bool issues = lw < NB;
        // Loads complete in order within a wave: with at most the loads of the `after` tiles requested last
        // outstanding, everything requested before them has landed.
        auto landed_but = [&](int after) {
            if (!issues || after <= 0) wait_vmcnt<0>();
            else if (after == 1) wait_vmcnt<LPT>();
            else if (after == 2) wait_vmcnt<2 * LPT>();
            else if (after == 3) wait_vmcnt<3 * LPT>();
            else wait_vmcnt<4 * LPT>();
        };
        auto tiles_in = [&](int first, int last) { return max(0, min(NT - 1, last) - first + 1); };
        wait_vmcnt<0>();
        __syncthreads();                                    // phase 0 has landed
        __syncthreads();                                    // the pixel region is free
        for (int p = 1; p < NPAIR; ++p) request_pair(p);
        for (int j = 0; j < NP; ++j) {
            // Tick j works on pair j; pair j + 1 must have landed when it ends.  Pair j + NPAIR - 1 takes the slots
            // of pair j - 1, which every compute wave has left at the last barrier.
            if (j >= 1) request_pair(j + NPAIR - 1);
            landed_but(tiles_in(2 * (j + 2), 2 * (j + NPAIR - 1) + 1));
            __syncthreads();
        }
        return;
    }

    // =========================== compute waves ==============================================
    const int team = wave >> 2;
    const int wq = wave & 3;
    const int frow = lane & 31, fk = lane >> 5;
    const char* lds_b = reinterpret_cast<const char*>(lds);
    const int arow = wq * 32 + frow;
    const uint32_t a_base = (uint32_t)(arow * PITCH + (swz<CPR>(arow, fk) << 4));
    const uint32_t b_base = (uint32_t)(frow * PITCH + (swz<CPR>(frow, fk) << 4));
    char* dep = reinterpret_cast<char*>(lds) + LY::STG + team * (kPwsStaging / 2);
    const uint32_t dep0 = stage_off(arow, fk);

    floatx16 acc;
    frag_t areg[KK];
    // Filter fragments are read two K slices ahead.
    auto multiply = [&](int slot) {
        const char* pb = lds_b + LY::slot(slot);
        constexpr int AHEAD = 2;
        frag_t b[AHEAD];
#pragma unroll
        for (int kk = 0; kk < AHEAD; ++kk) b[kk] = *reinterpret_cast<const frag_t*>(pb + (b_base ^ (uint32_t)(kk << 5)));
#pragma unroll
        for (int kk = 0; kk < KK; ++kk) {
            if (kk == 0) {
                floatx16 z;
#pragma unroll
                for (int v = 0; v < 16; ++v) z[v] = 0.f;
                acc = Elem<T>::mfma32(b[kk % AHEAD], areg[kk], z);
            } else {
                acc = Elem<T>::mfma32(b[kk % AHEAD], areg[kk], acc);
            }
            if (kk + AHEAD < KK)
                b[kk % AHEAD] = *reinterpret_cast<const frag_t*>(pb + (b_base ^ (uint32_t)((kk + AHEAD) << 5)));
        }
    };

    wait_vmcnt<0>();
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < KK; ++kk) areg[kk] = *reinterpret_cast<const frag_t*>(lds_b + (a_base ^ (uint32_t)(kk << 5)));
    __syncthreads();                                        // (waits for the reads above)
    for (int j = 0; j < NP; ++j) {
        const int tile = 2 * j + team;
        if (tile < NT) {
            multiply(tile % LY::SLOTS);
            // lane l holds pixel l%32 of the wave's fragment and, in element v, filter 8*(v/4) + 4*(l/32) + v%4:
            // piece 2*(v/4) + l/32 of the pixel's staging row, i.e. the lane's address xor (v/4 << 5)
            char* area = dep + (j & 1) * kPwsStaging;
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                floatx4 v = {acc[4 * gq], acc[4 * gq + 1], acc[4 * gq + 2], acc[4 * gq + 3]};
                *reinterpret_cast<floatx4*>(area + (dep0 ^ (uint32_t)(gq << 5))) = v;
            }
        }
        __syncthreads();
    }
}

bool plan_pw(const ConvShape& s, PwGeom* g) {
    if (s.R != 1 || s.S != 1) return false;
    if (s.C != 64 && s.C != 128 && s.C != 256) return false;
    if ((s.K & 3) || s.P >= (1 << 14) || s.Q >= (1 << 14)) return false;
    if ((long)s.K * s.C * 2 >= (1L << 31)) return false;
    // pixels of one workgroup span at most 128 / PQ + 2 images; their bytes are addressed with 31 bits
    const long img_bytes = (long)s.H * s.W * s.C * 2;
    if ((kPwBM / s.PQ + 2) * img_bytes >= (1L << 31)) return false;
    if ((long)kPwBM * s.K * 4 >= (1L << 31)) return false;
    const long cus = device_cus();
    const long rounds = (s.M + cus * kPwBM - 1) / (cus * kPwBM);
    long nwg = cus * rounds;
    if (nwg > s.M) nwg = s.M;
    const long rows = (s.M + nwg - 1) / nwg;                 // <= 128
    g->rows_per_wg = (int)rows;
    g->tiles_n = (s.K + kPwBN - 1) / kPwBN;
    g->inv_q = 1.0f / (float)s.Q;
    g->inv_p = 1.0f / (float)s.P;
    return true;
}

template <typename T, typename TO, int CPR, int FORM>
hipError_t launch_pw_t(const void* x, const void* w, void* y, const ConvShape& s, const PwGeom& g, hipStream_t st) {
    // FORM 0: staging of 2 KiB per compute wave; FORM 1: two staging areas for the store waves
    constexpr int lds_bytes = FORM == 0 ? (kPwBM + 4 * kPwBN) * CPR * 16 + 8 * kPwStage : PwsLayout<CPR>::LDS_BYTES;
    static_assert(lds_bytes <= 160 * 1024, "LDS of a compute unit");
    auto kern = FORM == 0 ? ipw_kernel<T, TO, CPR> : ipws_kernel<T, TO, CPR>;
    static std::atomic<bool> raised{false};
    if (!raised.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes);
        if (e != hipSuccess) return e;
        raised.store(true, std::memory_order_release);
    }
    const int nwg = (s.M + g.rows_per_wg - 1) / g.rows_per_wg;
    hipLaunchKernelGGL(kern, dim3((unsigned)nwg), dim3(kPwWaves * 64), lds_bytes, st, (const T*)x, (const T*)w, (TO*)y, s, g);
    return hipGetLastError();
}

template <typename T, typename TO, int FORM>
hipError_t launch_pw_c(const void* x, const void* w, void* y, const ConvShape& s, const PwGeom& g, hipStream_t st) {
    switch (s.C) {
        case 64: return launch_pw_t<T, TO, 8, FORM>(x, w, y, s, g, st);
        case 128: return launch_pw_t<T, TO, 16, FORM>(x, w, y, s, g, st);
        case 256: return launch_pw_t<T, TO, 32, FORM>(x, w, y, s, g, st);
        default: return hipErrorInvalidConfiguration;
    }
}

template <int FORM>
hipError_t launch_pw_f(const void* x, const void* w, void* y, const ConvShape& s, const PwGeom& g, int in_t, int out_t, hipStream_t st) {
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_pw_c<bf16_t, float, FORM>(x, w, y, s, g, st);
        if (out_t == OUT_BF16) return launch_pw_c<bf16_t, bf16_t, FORM>(x, w, y, s, g, st);
    } else if (in_t == IN_F16) {
        if (out_t == OUT_F32) return launch_pw_c<f16_t, float, FORM>(x, w, y, s, g, st);
        if (out_t == OUT_F16) return launch_pw_c<f16_t, f16_t, FORM>(x, w, y, s, g, st);
    }
    return hipErrorInvalidConfiguration;
}

const char* const kPwNames[] = {"a128x32_2x4+8", "a128x32_2x4+4+4"};
constexpr int kNumPw = 2;

}  // namespace

bool pointwise_supported(const ConvShape& s) {
    PwGeom g;
    return plan_pw(s, &g);
}

// Where these kernels measured faster than the per-tap kernels (28x28 and 56x56 maps, 64 to 256 channels, 128 to
// 1024 filters, batch 16 to 128, with the output stores written through).  The MFMAs always run on 128 rows and
// every workgroup streams all filters, so a workgroup needs enough pixels: 96 of 128 for the first form, 64 (48 at
// 128 channels) for the form with store waves, which loses less when the tile is not full (its stores, not its
// MFMAs, set the pace).  At 64 channels three workgroups of the first form share a compute unit, at 128 channels
// two, and that overlaps as well as store waves do up to 512 filters; beyond, and at 256 channels (one workgroup
// per compute unit either way), the store waves win (-3 to -12 %).  With 256 channels in several rounds of
// workgroups the per-tap kernel with 256-row tiles is faster up to 256 filters.
// Returns the variant (0: compute waves store, 1: store waves) or -1.
int pointwise_choose(const ConvShape& s) {
    PwGeom g;
    if (!plan_pw(s, &g)) return -1;
    const long nwg = (s.M + g.rows_per_wg - 1) / g.rows_per_wg;
    const bool one_round = nwg <= device_cus();
    if (s.C == 64) return g.rows_per_wg >= 96 ? 0 : -1;
    if (s.C == 128) {
        if (g.rows_per_wg < 48) return -1;
        return g.rows_per_wg >= 96 && s.K <= 512 ? 0 : 1;
    }
    if (g.rows_per_wg < 64) return -1;
    if (one_round) return 1;
    return s.K >= 512 ? 1 : -1;
}

int pointwise_num_variants() { return kNumPw; }
const char* pointwise_variant_name(int v) { return kPwNames[v]; }

hipError_t launch_pointwise(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v, hipStream_t st) {
    PwGeom g;
    if (!plan_pw(s, &g)) return hipErrorInvalidConfiguration;
    if (v == 0) return launch_pw_f<0>(x, w, y, s, g, in_t, out_t, st);
    if (v == 1) return launch_pw_f<1>(x, w, y, s, g, in_t, out_t, st);
    return hipErrorInvalidValue;
}

}  // namespace iconv

// Channel-last implicit im2col (paper sections 2.3 and 3.1): the lowered matrix's columns are
// ordered channel, tap row, tap column (channel slowest) over an NCHW input and KCRS filters, the
// order of the conventional implicit-GEMM convolution that the paper's channel-first design is
// measured against.  Built only as the second in-run comparison of the stride study: with this
// order the elements of one lowered column that neighbouring output pixels need lie `stride`
// input pixels apart, so the gather that feeds the A tile reads 1/stride of every cache line it
// touches, and the filter taps of one K step land on different input rows.
//
// Same block-level GEMM as the channel-first kernels (one workgroup per 128 x 128 output tile,
// 32x32x16 MFMA, fp32 accumulators, y in NPQK), but the A tile is gathered element by element:
// thread t < 128 owns tile row t (one output pixel) and fetches its 32 lowered elements of the K
// step with 2-byte loads (coalesced across the threads of a wave along the pixel index when the
// stride is 1), packs them and writes the row to LDS; threads 128..255 bring in the filter tile.
// Global loads of step i + 1 are issued before the MFMAs of step i (register staging).
#include "iconv_common.h"
#include "iconv_device.h"

namespace iconv {

namespace {

constexpr int kClBM = 128, kClBN = 128, kClBK = 32;

template <typename T, typename TO>
__global__ void __launch_bounds__(256)
chlast_kernel(const T* __restrict__ x, const T* __restrict__ w, TO* __restrict__ y, const ConvShape s, const int tiles_n) {
    constexpr int BM = kClBM, BN = kClBN, BK = kClBK;
    constexpr int CPR = BK / 8;                 // 16-byte chunks per tile row
    constexpr int MI = 2, NI = 2, KI = BK / 16; // four waves of 64 x 64
    typedef typename Elem<T>::frag frag_t;
    typedef uint16_t raw_t;                     // bf16 and fp16 both travel as 16 raw bits

    __shared__ u32x4 lds[(BM + BN) * CPR];      // [A: BM rows x CPR chunks][B: BN rows x CPR chunks]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave >> 1, wave_n = wave & 1;
    const int tile_n = blockIdx.x % tiles_n, tile_m = blockIdx.x / tiles_n;
    const int m0 = tile_m * BM, k0 = tile_n * BN;
    const raw_t* xr = reinterpret_cast<const raw_t*>(x);
    const raw_t* wr = reinterpret_cast<const raw_t*>(w);

    // ---- loader state
    const bool a_thread = tid < BM;
    const int row = a_thread ? tid : tid - BM;  // tile row this thread fills (A: pixel, B: filter)
    int a_h0 = -(1 << 28), a_w0 = 0;            // input coordinates of tap (0, 0); never in bounds for rows past M
    long a_base = 0;                            // element offset of (n, channel 0, a_h0, a_w0)
    long b_base = -1;                           // element offset of the filter's first lowered element, -1 past K
    if (a_thread) {
        const int m = m0 + row;
        if (m < s.M) {
            const int n = m / s.PQ;
            const int pq = m - n * s.PQ;
            const int p = pq / s.Q, q = pq - p * s.Q;
            a_h0 = p * s.stride - s.pad;
            a_w0 = q * s.stride - s.pad;
            a_base = ((long)n * s.C * s.H + a_h0) * s.W + a_w0;
        }
    } else if (k0 + row < s.K) {
        b_base = (long)(k0 + row) * s.Kg;
    }
    const bool b_vec = (s.Kg & 7) == 0;         // filter rows are then made of whole, aligned 16-byte chunks
    const long plane = (long)s.H * s.W;

    const int steps = (s.Kg + BK - 1) / BK;
    // Fetches this thread's 32 elements of K step `step` into four packed 16-byte chunks.
    auto fetch = [&](int step, u32x4 (&out)[CPR]) __attribute__((always_inline)) {
        const int kbeg = step * BK;
        if (a_thread) {
            // lowered column kbeg + j = (c, r, s): wave-uniform, walked incrementally
            int c = kbeg / (s.R * s.S);
            int rs = kbeg - c * (s.R * s.S);
            int r = rs / s.S, ss = rs - r * s.S;
#pragma unroll
            for (int ch = 0; ch < CPR; ++ch) {
                uint32_t packed[4];
#pragma unroll
                for (int e = 0; e < 8; ++e) {
                    const int dh = r * s.dil, dw = ss * s.dil;
                    const bool ok = (kbeg + ch * 8 + e) < s.Kg && (unsigned)(a_h0 + dh) < (unsigned)s.H &&
                                    (unsigned)(a_w0 + dw) < (unsigned)s.W;
                    const long off = a_base + c * plane + (long)dh * s.W + dw;
                    const uint32_t v = ok ? (uint32_t)xr[off] : 0u;
                    if (e & 1) packed[e >> 1] |= v << 16; else packed[e >> 1] = v;
                    if (++ss == s.S) { ss = 0; if (++r == s.R) { r = 0; ++c; } }
                }
                out[ch] = u32x4{packed[0], packed[1], packed[2], packed[3]};
            }
        } else {
#pragma unroll
            for (int ch = 0; ch < CPR; ++ch) {
                const int kk = kbeg + ch * 8;
                if (b_base >= 0 && b_vec && kk + 8 <= s.Kg) {
                    out[ch] = *reinterpret_cast<const u32x4*>(wr + b_base + kk);
                } else {
                    uint32_t packed[4] = {0u, 0u, 0u, 0u};
#pragma unroll
                    for (int e = 0; e < 8; ++e) {
                        const uint32_t v = (b_base >= 0 && kk + e < s.Kg) ? (uint32_t)wr[b_base + kk + e] : 0u;
                        packed[e >> 1] |= (e & 1) ? v << 16 : v;
                    }
                    out[ch] = u32x4{packed[0], packed[1], packed[2], packed[3]};
                }
            }
        }
    };
    // Writes the staged row to LDS (chunk swizzle as in the channel-first kernels).
    auto deposit = [&](const u32x4 (&in)[CPR]) __attribute__((always_inline)) {
        u32x4* dst = lds + (a_thread ? 0 : BM * CPR) + row * CPR;
#pragma unroll
        for (int ch = 0; ch < CPR; ++ch) dst[swz<CPR>(row, ch)] = in[ch];
    };

    floatx16 acc[MI][NI];
#pragma unroll
    for (int mi = 0; mi < MI; ++mi)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    const int frow = lane & 31, fk = lane >> 5;
    u32x4 staged[CPR];
    fetch(0, staged);
    for (int step = 0; step < steps; ++step) {
        __syncthreads();                        // the previous step's fragments have been read
        deposit(staged);
        __syncthreads();
        if (step + 1 < steps) fetch(step + 1, staged);
        const u32x4* A = lds;
        const u32x4* Bt = lds + BM * CPR;
#pragma unroll
        for (int kk = 0; kk < KI; ++kk) {
            frag_t af[MI], bfr[NI];
#pragma unroll
            for (int mi = 0; mi < MI; ++mi) {
                const int r = wave_m * 64 + mi * 32 + frow;
                af[mi] = __builtin_bit_cast(frag_t, A[r * CPR + swz<CPR>(r, kk * 2 + fk)]);
            }
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
                const int r = wave_n * 64 + ni * 32 + frow;
                bfr[ni] = __builtin_bit_cast(frag_t, Bt[r * CPR + swz<CPR>(r, kk * 2 + fk)]);
            }
#pragma unroll
            for (int mi = 0; mi < MI; ++mi)
#pragma unroll
                for (int ni = 0; ni < NI; ++ni) acc[mi][ni] = Elem<T>::mfma32(bfr[ni], af[mi], acc[mi][ni]);
        }
    }

    // ---- epilogue: as in the channel-first per-tap kernel (lane l holds pixel l%32 and, in element v,
    // filter 8*(v/4) + 4*(l/32) + v%4 of the 32-wide block)
    const bool vec_ok = (s.K & 3) == 0;
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
        const int m = m0 + wave_m * 64 + mi * 32 + frow;
        if (m < s.M) {
            TO* yrow = y + (size_t)m * s.K;
#pragma unroll
            for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
                for (int gq = 0; gq < 4; ++gq) {
                    const int col = k0 + wave_n * 64 + ni * 32 + 8 * gq + 4 * fk;
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

template <typename T, typename TO>
hipError_t launch_cl(const void* x, const void* w, void* y, const ConvShape& s, hipStream_t st) {
    const int tiles_m = (s.M + kClBM - 1) / kClBM, tiles_n = (s.K + kClBN - 1) / kClBN;
    hipLaunchKernelGGL((chlast_kernel<T, TO>), dim3((unsigned)(tiles_m * tiles_n)), dim3(256), 0, st, (const T*)x, (const T*)w,
                       (TO*)y, s, tiles_n);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_channel_last(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, hipStream_t st) {
    if (in_t == IN_BF16) {
        if (out_t == OUT_F32) return launch_cl<bf16_t, float>(x, w, y, s, st);
        return launch_cl<bf16_t, bf16_t>(x, w, y, s, st);
    }
    if (out_t == OUT_F32) return launch_cl<f16_t, float>(x, w, y, s, st);
    return launch_cl<f16_t, f16_t>(x, w, y, s, st);
}

}  // namespace iconv

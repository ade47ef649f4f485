// Plain (non-MFMA) kernels: the direct convolution fallback, the explicit lowering kernel and
// the copy probe.
#include "iconv_common.h"

namespace iconv {

namespace {

template <typename T> __device__ __forceinline__ float ld(const T* p) { return (float)*p; }

// Direct convolution, one thread per output element, fp32 FMA in (r, s, c) order.
// Lanes run along k, so x reads are wave-uniform broadcasts.  Used for fp32 inputs and for
// channel counts the MFMA paths do not take; correctness path, not a fast one.
template <typename TI, typename TO>
__global__ void __launch_bounds__(256) direct_kernel(const TI* __restrict__ x, const TI* __restrict__ w,
                                                    TO* __restrict__ y, ConvShape s) {
    const long long total = (long long)s.M * s.K;
    const long long stride_t = (long long)gridDim.x * blockDim.x;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride_t) {
        const int k = (int)(idx % s.K);
        const int m = (int)(idx / s.K);
        const int n = m / s.PQ;
        const int pq = m - n * s.PQ;
        const int p = pq / s.Q, q = pq - p * s.Q;
        const int h0 = p * s.stride - s.pad, w0 = q * s.stride - s.pad;
        float acc = 0.f;
        for (int r = 0; r < s.R; ++r) {
            const int h = h0 + r * s.dil;
            if ((unsigned)h >= (unsigned)s.H) continue;
            for (int ss = 0; ss < s.S; ++ss) {
                const int ww = w0 + ss * s.dil;
                if ((unsigned)ww >= (unsigned)s.W) continue;
                const TI* xp = x + ((size_t)((size_t)n * s.H + h) * s.W + ww) * s.C;
                const TI* wp = w + ((size_t)((size_t)k * s.R + r) * s.S + ss) * s.C;
                // (unrolled so that the loads of several channels are in flight at once; the sum
                // itself stays one chain in channel order)
#pragma unroll 8
                for (int c = 0; c < s.C; ++c) acc = fmaf(ld(xp + c), ld(wp + c), acc);
            }
        }
        y[idx] = to_out<TO>(acc);
    }
}

// Explicit im2col (paper section 2.1): lowered[m][(r*S+s)*C + c], zero where the tap falls
// outside the map; rows are `pitch` elements long (Kg rounded up for the MFMA GEMM) and the tail
// of a row is zero.  One thread per (output pixel, VEC-element piece of the channel run): it decodes
// the pixel once and walks all R*S taps, so the index arithmetic is paid once per R*S pieces moved.
// V: the piece type (16, 8, 4 or 2 bytes), cv pieces per pixel.
template <typename V>
__global__ void __launch_bounds__(256) im2col_kernel(const V* __restrict__ x, V* __restrict__ low, ConvShape s, int cv, int pitch_v) {
    const long long total = (long long)s.M * cv;
    const long long stride_t = (long long)gridDim.x * blockDim.x;
    const int RS = s.R * s.S;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride_t) {
        const int m = (int)(idx / cv);
        const int c = (int)(idx - (long long)m * cv);
        const int n = m / s.PQ;
        const int pq = m - n * s.PQ;
        const int p = pq / s.Q, q = pq - p * s.Q;
        const int h0 = p * s.stride - s.pad, w0 = q * s.stride - s.pad;
        const V* xn = x + (size_t)n * s.H * s.W * cv + c;
        V* row = low + (size_t)m * pitch_v + c;
        for (int r = 0; r < s.R; ++r) {
            const int h = h0 + r * s.dil;
            for (int ss = 0; ss < s.S; ++ss) {
                const int ww = w0 + ss * s.dil;
                V v = {};
                if ((unsigned)h < (unsigned)s.H && (unsigned)ww < (unsigned)s.W) v = xn[((size_t)h * s.W + ww) * cv];
                row[(size_t)(r * s.S + ss) * cv] = v;
            }
        }
        // zero tail of the row (pitch beyond R*S*C), split over the pixel's threads
        for (int t = RS * cv + c; t < pitch_v; t += cv) low[(size_t)m * pitch_v + t] = V{};
    }
}

// The same for pixels of few pieces (cv < 4, e.g. four 16-bit channels = one 8-byte piece): one thread per
// (output pixel, tap), taps fastest, so that the threads of a wave write one contiguous stretch of a lowered row.
template <typename V>
__global__ void __launch_bounds__(256) im2col_taps_kernel(const V* __restrict__ x, V* __restrict__ low, ConvShape s, int cv, int pitch_v) {
    const int RS = s.R * s.S;
    const int per_row = RS + (pitch_v - RS * cv + cv - 1) / cv;      // taps, then the zero tail in tap-sized steps
    const long long total = (long long)s.M * per_row;
    const long long stride_t = (long long)gridDim.x * blockDim.x;
    for (long long idx = (long long)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride_t) {
        const int m = (int)(idx / per_row);
        const int tap = (int)(idx - (long long)m * per_row);
        V* dst = low + (size_t)m * pitch_v + (size_t)tap * cv;
        if (tap >= RS) {
            for (int c = 0; c < cv && tap * cv + c < pitch_v; ++c) dst[c] = V{};
            continue;
        }
        const int n = m / s.PQ;
        const int pq = m - n * s.PQ;
        const int p = pq / s.Q, q = pq - p * s.Q;
        const int r = tap / s.S, ss = tap - r * s.S;
        const int h = p * s.stride - s.pad + r * s.dil, ww = q * s.stride - s.pad + ss * s.dil;
        const bool ok = (unsigned)h < (unsigned)s.H && (unsigned)ww < (unsigned)s.W;
        const V* src = x + ((size_t)((size_t)n * s.H + h) * s.W + ww) * cv;
        for (int c = 0; c < cv; ++c) dst[c] = ok ? src[c] : V{};
    }
}

// Filter matrix K x Kg copied into rows of `pitch` elements with a zero tail (the GEMM operand of the
// explicit variant when Kg is not a multiple of eight elements).
__global__ void __launch_bounds__(256) pad_rows_kernel(const uint16_t* __restrict__ src, uint16_t* __restrict__ dst, int rows,
                                                      int len, int pitch) {
    const long long total = (long long)rows * pitch;
    for (long long i = (long long)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (long long)gridDim.x * blockDim.x) {
        const int r = (int)(i / pitch), k = (int)(i - (long long)r * pitch);
        dst[i] = k < len ? src[(size_t)r * len + k] : (uint16_t)0;
    }
}

__global__ void __launch_bounds__(256) copy_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
    const size_t stride_t = (size_t)gridDim.x * blockDim.x;
    for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride_t) dst[i] = src[i];
}

// Register-only MFMA loop: eight independent accumulator tiles per wave, operands never reloaded.
// RANDOM = false: one small-integer operand pair for all MFMAs (few bits toggle between
// instructions); RANDOM = true: four operand pairs of pseudo-random values in +-[0.5, 1), a
// different pair on consecutive MFMAs, which is what real data does to the multiplier inputs.
template <bool RANDOM>
__global__ void __launch_bounds__(256) mfma_probe_kernel(float* __restrict__ out, int iters) {
    floatx16 acc[8];
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[i][v] = 0.f;
    bf16x8 a[4], b[4];
#pragma unroll
    for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            if (RANDOM) {
                uint32_t h = (uint32_t)(blockIdx.x * 256 + threadIdx.x) * 2654435761u + (uint32_t)(r * 8 + j) * 40503u;
                h ^= h >> 15; h *= 2246822519u; h ^= h >> 13;
                const uint16_t ua = (uint16_t)((h & 0x807fu) | 0x3f00u), ub = (uint16_t)(((h >> 16) & 0x807fu) | 0x3f00u);
                a[r][j] = __builtin_bit_cast(bf16_t, ua);
                b[r][j] = __builtin_bit_cast(bf16_t, ub);
            } else {
                a[r][j] = (bf16_t)(float)((threadIdx.x + j) & 7);
                b[r][j] = (bf16_t)(float)(j + 1);
            }
        }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[RANDOM ? (i & 3) : 0], b[RANDOM ? ((i >> 1) & 3) : 0], acc[i], 0, 0, 0);
    }
    float sum = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int v = 0; v < 16; ++v) sum += acc[i][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = sum;
}

int grid_for(long long total, int block) {
    long long g = (total + block - 1) / block;
    const long long cap = 256LL * 64;  // grid-stride beyond this
    if (g > cap) g = cap;
    if (g < 1) g = 1;
    return (int)g;
}

template <typename TI>
hipError_t direct_out(const void* x, const void* w, void* y, const ConvShape& s, int out_t, hipStream_t st) {
    const int grid = grid_for((long long)s.M * s.K, 256);
    switch (out_t) {
        case OUT_F32:
            hipLaunchKernelGGL((direct_kernel<TI, float>), dim3(grid), dim3(256), 0, st, (const TI*)x, (const TI*)w,
                               (float*)y, s);
            break;
        case OUT_BF16:
            hipLaunchKernelGGL((direct_kernel<TI, bf16_t>), dim3(grid), dim3(256), 0, st, (const TI*)x, (const TI*)w,
                               (bf16_t*)y, s);
            break;
        default:
            hipLaunchKernelGGL((direct_kernel<TI, f16_t>), dim3(grid), dim3(256), 0, st, (const TI*)x, (const TI*)w,
                               (f16_t*)y, s);
            break;
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_direct(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t,
                         hipStream_t st) {
    switch (in_t) {
        case IN_F32: return direct_out<float>(x, w, y, s, out_t, st);
        case IN_BF16: return direct_out<bf16_t>(x, w, y, s, out_t, st);
        default: return direct_out<f16_t>(x, w, y, s, out_t, st);
    }
}

hipError_t launch_im2col(const void* x, void* low, const ConvShape& s, int elt_bytes, int pitch_elems, hipStream_t st) {
    const int cbytes = s.C * elt_bytes;  // bytes of one pixel's channel run
    const long long pitch_bytes = (long long)pitch_elems * elt_bytes;
    // the widest piece that divides both the channel run and the row pitch
    int piece = 16;
    while (piece > elt_bytes && ((cbytes % piece) != 0 || (pitch_bytes % piece) != 0)) piece >>= 1;
    const int cv = cbytes / piece, pitch_v = (int)(pitch_bytes / piece);
    if (cv < 4) {
        const int RS = s.R * s.S;
        const int grid = grid_for((long long)s.M * (RS + (pitch_v - RS * cv + cv - 1) / cv), 256);
        switch (piece) {
            case 16: hipLaunchKernelGGL(im2col_taps_kernel<uint4>, dim3(grid), dim3(256), 0, st, (const uint4*)x, (uint4*)low, s, cv, pitch_v); break;
            case 8: hipLaunchKernelGGL(im2col_taps_kernel<uint2>, dim3(grid), dim3(256), 0, st, (const uint2*)x, (uint2*)low, s, cv, pitch_v); break;
            case 4: hipLaunchKernelGGL(im2col_taps_kernel<uint32_t>, dim3(grid), dim3(256), 0, st, (const uint32_t*)x, (uint32_t*)low, s, cv, pitch_v); break;
            default: hipLaunchKernelGGL(im2col_taps_kernel<uint16_t>, dim3(grid), dim3(256), 0, st, (const uint16_t*)x, (uint16_t*)low, s, cv, pitch_v); break;
        }
        return hipGetLastError();
    }
    const int grid = grid_for((long long)s.M * cv, 256);
    switch (piece) {
        case 16: hipLaunchKernelGGL(im2col_kernel<uint4>, dim3(grid), dim3(256), 0, st, (const uint4*)x, (uint4*)low, s, cv, pitch_v); break;
        case 8: hipLaunchKernelGGL(im2col_kernel<uint2>, dim3(grid), dim3(256), 0, st, (const uint2*)x, (uint2*)low, s, cv, pitch_v); break;
        case 4: hipLaunchKernelGGL(im2col_kernel<uint32_t>, dim3(grid), dim3(256), 0, st, (const uint32_t*)x, (uint32_t*)low, s, cv, pitch_v); break;
        default: hipLaunchKernelGGL(im2col_kernel<uint16_t>, dim3(grid), dim3(256), 0, st, (const uint16_t*)x, (uint16_t*)low, s, cv, pitch_v); break;
    }
    return hipGetLastError();
}

hipError_t launch_pad_rows(const void* src, void* dst, int rows, int len, int pitch, hipStream_t st) {
    hipLaunchKernelGGL(pad_rows_kernel, dim3(grid_for((long long)rows * pitch, 256)), dim3(256), 0, st, (const uint16_t*)src,
                       (uint16_t*)dst, rows, len, pitch);
    return hipGetLastError();
}

hipError_t launch_mfma_probe(void* out, int iters, bool random_operands, hipStream_t st) {
    if (random_operands)
        hipLaunchKernelGGL(mfma_probe_kernel<true>, dim3(kMfmaProbeGroups), dim3(256), 0, st, (float*)out, iters);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<false>, dim3(kMfmaProbeGroups), dim3(256), 0, st, (float*)out, iters);
    return hipGetLastError();
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st) {
    const size_t n16 = bytes / 16;
    hipLaunchKernelGGL(copy_kernel, dim3(grid_for((long long)n16, 256)), dim3(256), 0, st, (const uint4*)src,
                       (uint4*)dst, n16);
    return hipGetLastError();
}

}  // namespace iconv

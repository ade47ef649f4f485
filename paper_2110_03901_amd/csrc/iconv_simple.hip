// Plain (non-MFMA) kernels: the direct convolution fallback, the explicit lowering kernels and
// the copy, MFMA and LDS probes.
#include "iconv_common.h"
#include "iconv_device.h"

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

// The same copy with the stores of the convolution kernels' epilogues: whole lines per instruction, written through
// (kStoreYPolicy).  For destinations below 4 GiB (one buffer descriptor).
__global__ void __launch_bounds__(256) copy_wt_kernel(const uint4* __restrict__ src, uint4* __restrict__ dst, uint32_t n16) {
    const rsrc_t d_rsrc = __builtin_amdgcn_make_buffer_rsrc(dst, 0, n16 * 16u, kRsrcFlags);
    const uint32_t stride_t = gridDim.x * blockDim.x;
    for (uint32_t i = blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += stride_t) {
        const uint4 v = src[i];
        __builtin_amdgcn_raw_buffer_store_b128(u32x4{v.x, v.y, v.z, v.w}, d_rsrc, (int)(i * 16u), 0, kStoreYPolicy);
    }
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

// LDS access-pattern probe: every wave issues `iters` x 8 ds_read_b128 (or ds_write_b128) of one fixed
// 64-lane address pattern on a 6 KiB region of its own, nothing else in the loop.  Patterns:
//   0  read, lane-linear (lane l at byte 16*l): the conflict-free reference
//   1  write, lane-linear
//   2  read, MFMA operand shape (lane l: tile row l%32, chunk l/32) on 64-byte rows, no swizzle
//   3  the same through swz<4>, the layout of the kernels' 64-byte rows
//   4  the same on 128-byte rows through swz<8>
//   5  write, the deposit of store_frag_staged: lanes of 16 pixels (half the wave) write piece
//      2*gq + l/32 of pixel l%16 at stage_off(pixel, piece), gq = 0..3
//   6  write, the deposit of the merged-tap kernel: all 64 lanes, 32 pixels, the same layout
//   7  write, 32 pixels, piece c of pixel i at i*128 + ((c ^ (i>>1 & 7)) << 4): a layout that is free of
//      conflicts for reads but puts two lanes of every write pass on the same banks (reference)
// Timed, it gives the cycles an LDS instruction costs a compute unit; under a counter pass it shows
// what SQ_LDS_BANK_CONFLICT reads for accesses whose conflicts are known.
template <int PATTERN>
__global__ void __launch_bounds__(256) lds_probe_kernel(float* __restrict__ out, int iters) {
    __shared__ u32x4 buf[4 * 384];
    for (int i = threadIdx.x; i < 4 * 384; i += 256) buf[i] = u32x4{(uint32_t)i, 1u, 2u, 3u};
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int row = lane & 31, chunk = lane >> 5;
    uint32_t byte;
    if (PATTERN <= 1) byte = (uint32_t)lane * 16u;
    else if (PATTERN == 2) byte = (uint32_t)(row * 64 + chunk * 16);
    else if (PATTERN == 3) byte = (uint32_t)(row * 64 + swz<4>(row, chunk) * 16);
    else if (PATTERN == 4) byte = (uint32_t)(row * 128 + swz<8>(row, chunk) * 16);
    else if (PATTERN == 5) byte = stage_off(row & 15, chunk);
    else if (PATTERN == 6) byte = stage_off(row, chunk);
    else byte = (uint32_t)(row * 128 + ((chunk ^ ((row >> 1) & 7)) << 4));
    // at most 31 * 128 + 7 * 16 + 16 bytes of pattern + 1792 bytes of instruction offsets = 5888 < 6144
    const uint32_t addr = (uint32_t)(size_t)(__attribute__((address_space(3))) void*)buf + (uint32_t)wave * 6144u + byte;
    u32x4 sum = {0u, 0u, 0u, 0u};
    for (int it = 0; it < iters; ++it) {
        if (PATTERN >= 5) {
            // pieces 2*gq + chunk: the address xor (gq << 5); two rounds, the second 2 KiB further on
            const u32x4 v = {(uint32_t)it, (uint32_t)lane, 2u, 3u};
            if (PATTERN >= 6 || row < 16)
                asm volatile("ds_write_b128 %0, %4\n\tds_write_b128 %1, %4\n\tds_write_b128 %2, %4\n\tds_write_b128 %3, %4\n\t"
                             "ds_write_b128 %0, %4 offset:2048\n\tds_write_b128 %1, %4 offset:2048\n\t"
                             "ds_write_b128 %2, %4 offset:2048\n\tds_write_b128 %3, %4 offset:2048\n\ts_waitcnt lgkmcnt(0)"
                             :
                             : "v"(addr), "v"(addr ^ 32u), "v"(addr ^ 64u), "v"(addr ^ 96u), "v"(v)
                             : "memory");
        } else if (PATTERN == 1) {
            const u32x4 v = {(uint32_t)it, (uint32_t)lane, 2u, 3u};
            asm volatile("ds_write_b128 %0, %1\n\tds_write_b128 %0, %1 offset:256\n\tds_write_b128 %0, %1 offset:512\n\t"
                         "ds_write_b128 %0, %1 offset:768\n\tds_write_b128 %0, %1 offset:1024\n\tds_write_b128 %0, %1 offset:1280\n\t"
                         "ds_write_b128 %0, %1 offset:1536\n\tds_write_b128 %0, %1 offset:1792\n\ts_waitcnt lgkmcnt(0)"
                         :
                         : "v"(addr), "v"(v)
                         : "memory");
        } else {
            u32x4 r0, r1, r2, r3, r4, r5, r6, r7;
            asm volatile("ds_read_b128 %0, %8\n\tds_read_b128 %1, %8 offset:256\n\tds_read_b128 %2, %8 offset:512\n\t"
                         "ds_read_b128 %3, %8 offset:768\n\tds_read_b128 %4, %8 offset:1024\n\tds_read_b128 %5, %8 offset:1280\n\t"
                         "ds_read_b128 %6, %8 offset:1536\n\tds_read_b128 %7, %8 offset:1792\n\ts_waitcnt lgkmcnt(0)"
                         : "=&v"(r0), "=&v"(r1), "=&v"(r2), "=&v"(r3), "=&v"(r4), "=&v"(r5), "=&v"(r6), "=&v"(r7)
                         : "v"(addr)
                         : "memory");
            sum ^= r0 ^ r1 ^ r2 ^ r3 ^ r4 ^ r5 ^ r6 ^ r7;
        }
    }
    if (PATTERN == 1 || PATTERN >= 5) sum = buf[threadIdx.x];
    out[blockIdx.x * blockDim.x + threadIdx.x] = (float)(sum.x ^ sum.y ^ sum.z ^ sum.w);
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

hipError_t launch_lds_probe(void* out, int iters, int pattern, hipStream_t st) {
    const dim3 grid(kMfmaProbeGroups), block(256);
    switch (pattern) {
        case 0: hipLaunchKernelGGL(lds_probe_kernel<0>, grid, block, 0, st, (float*)out, iters); break;
        case 1: hipLaunchKernelGGL(lds_probe_kernel<1>, grid, block, 0, st, (float*)out, iters); break;
        case 2: hipLaunchKernelGGL(lds_probe_kernel<2>, grid, block, 0, st, (float*)out, iters); break;
        case 3: hipLaunchKernelGGL(lds_probe_kernel<3>, grid, block, 0, st, (float*)out, iters); break;
        case 4: hipLaunchKernelGGL(lds_probe_kernel<4>, grid, block, 0, st, (float*)out, iters); break;
        case 5: hipLaunchKernelGGL(lds_probe_kernel<5>, grid, block, 0, st, (float*)out, iters); break;
        case 6: hipLaunchKernelGGL(lds_probe_kernel<6>, grid, block, 0, st, (float*)out, iters); break;
        case 7: hipLaunchKernelGGL(lds_probe_kernel<7>, grid, block, 0, st, (float*)out, iters); break;
        default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

int lds_stage_offset(int pixel, int piece) { return (int)stage_off(pixel, piece); }

int lds_swizzle(int chunks_per_row, int row, int chunk) {
    switch (chunks_per_row) {
        case 4: return swz<4>(row, chunk);
        case 8: return swz<8>(row, chunk);
        case 16: return swz<16>(row, chunk);
        default: return swz<32>(row, chunk);
    }
}

hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t st, bool write_through) {
    const size_t n16 = bytes / 16;
    if (write_through && bytes < (1ull << 32)) {
        hipLaunchKernelGGL(copy_wt_kernel, dim3(grid_for((long long)n16, 256)), dim3(256), 0, st, (const uint4*)src,
                           (uint4*)dst, (uint32_t)n16);
    } else {
        hipLaunchKernelGGL(copy_kernel, dim3(grid_for((long long)n16, 256)), dim3(256), 0, st, (const uint4*)src,
                           (uint4*)dst, n16);
    }
    return hipGetLastError();
}

}  // namespace iconv

// Device-side helpers shared by the MFMA kernels (gfx950 only).
#pragma once
#include "iconv_common.h"

namespace iconv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;
// dword 3 of a raw buffer descriptor on gfx9: 32-bit data format, no swizzle, offsets checked
// against num_records in bytes
constexpr int kRsrcFlags = 0x00020000;

// 16-byte-chunk swizzle of a tile row: keeps both the row-contiguous writes of the loader and
// the column-of-rows ds_read_b128 of the MFMA operand fetch spread over all banks.
template <int CPR> __device__ __forceinline__ int swz(int row, int chunk) {
    constexpr int RP = (8 / CPR) > 0 ? (8 / CPR) : 1;  // tile rows per 128 bytes
    return chunk ^ (((row / RP) ^ (row >> 3)) & (CPR - 1));
}

// One wave-wide 16-bytes-per-lane load from a buffer straight into LDS: lane l's data lands at
// lds_addr + 16*l; an out-of-range offset writes zeros.  Inline assembly on purpose: the
// compiler then does not pair every later LDS read with a wait for all outstanding loads, and
// the kernels place their own s_waitcnt vmcnt(n).
__device__ __forceinline__ void dma16(rsrc_t rsrc, uint32_t voff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, 0 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc)
                 : "memory", "m0");
}

// The same with a wave-uniform byte offset `soff` added to the address through the instruction's
// scalar offset operand, so that a lane-constant `voff` needs no vector arithmetic per load.
// Callers keep voff + soff below 2^32 and pass in-range sums for every lane that is not meant to
// read zeros; a lane meant to read zeros carries voff >= the buffer size.
__device__ __forceinline__ void dma16s(rsrc_t rsrc, uint32_t voff, uint32_t soff, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
                 :
                 : "s"(lds_addr), "v"(voff), "s"(rsrc), "s"(soff)
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

// Four consecutive outputs (16-byte aligned for fp32, 8-byte for 16-bit types) in one store.
template <typename O> __device__ __forceinline__ void store4(O* p, float a, float b, float c, float d);
template <> __device__ __forceinline__ void store4<float>(float* p, float a, float b, float c, float d) {
    floatx4 v = {a, b, c, d};
    *reinterpret_cast<floatx4*>(p) = v;
}
template <> __device__ __forceinline__ void store4<bf16_t>(bf16_t* p, float a, float b, float c, float d) {
    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
    bf16x4 v = {to_out<bf16_t>(a), to_out<bf16_t>(b), to_out<bf16_t>(c), to_out<bf16_t>(d)};
    *reinterpret_cast<bf16x4*>(p) = v;
}
template <> __device__ __forceinline__ void store4<f16_t>(f16_t* p, float a, float b, float c, float d) {
    typedef f16_t f16x4 __attribute__((ext_vector_type(4)));
    f16x4 v = {(f16_t)a, (f16_t)b, (f16_t)c, (f16_t)d};
    *reinterpret_cast<f16x4*>(p) = v;
}

// Four consecutive fp32 results (one 16-byte staging piece) to a buffer, converted to the output
// type; an offset at or past the end of the buffer drops the store.
template <typename O> __device__ __forceinline__ void store_piece(u32x4 v, rsrc_t rsrc, uint32_t off);
template <> __device__ __forceinline__ void store_piece<float>(u32x4 v, rsrc_t rsrc, uint32_t off) {
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, (int)off, 0, 0);
}
template <> __device__ __forceinline__ void store_piece<bf16_t>(u32x4 v, rsrc_t rsrc, uint32_t off) {
    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const floatx4 f = __builtin_bit_cast(floatx4, v);
    const bf16x4 h = {to_out<bf16_t>(f[0]), to_out<bf16_t>(f[1]), to_out<bf16_t>(f[2]), to_out<bf16_t>(f[3])};
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, h), rsrc, (int)off, 0, 0);
}
template <> __device__ __forceinline__ void store_piece<f16_t>(u32x4 v, rsrc_t rsrc, uint32_t off) {
    typedef f16_t f16x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const floatx4 f = __builtin_bit_cast(floatx4, v);
    const f16x4 h = {(f16_t)f[0], (f16_t)f[1], (f16_t)f[2], (f16_t)f[3]};
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, h), rsrc, (int)off, 0, 0);
}

}  // namespace iconv

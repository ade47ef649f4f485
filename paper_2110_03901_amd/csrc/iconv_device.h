// Device-side helpers shared by the MFMA kernels (gfx950 only).
#pragma once
#include "iconv_common.h"

namespace iconv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef __amdgpu_buffer_rsrc_t rsrc_t;
// dword 3 of a raw buffer descriptor on gfx9: 32-bit data format, no swizzle, offsets checked
// against num_records in bytes
constexpr int kRsrcFlags = 0x00020000;

// 16-byte-chunk swizzle of a tile row of CPR chunks.  The loader writes rows contiguously (lane-linear
// LDS-DMA, always conflict-free); the MFMA operand fetch is a ds_read_b128 of 32 consecutive rows x
// one chunk per half-wave, which the LDS serves in passes of 16 lanes: lanes 0-3, 12-15, 20-27 and
// lanes 4-11, 16-19, 28-31 of each half-wave (measured on gfx950 by timing lane pairs that share a
// bank).  A pass is conflict-free when its 16 lanes hit 16 different 16-byte slots of the 256-byte
// bank window.  128-byte rows (and wider): XOR the row number, folded with row >> 3.  64-byte rows:
// four consecutive rows fill a window, so the term must be constant over them and differ between
// the four row quads of a pass (quads 0, 3, 5, 6 or 1, 2, 4, 7): the quad number's low two bits.
template <int CPR> __host__ __device__ __forceinline__ constexpr int swz(int row, int chunk) {
    if (CPR == 4) return chunk ^ ((row >> 2) & 3);
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

// Touches the first `BYTES` bytes of the kernel-argument segment, one scalar load per 64-byte line,
// all in flight at once, and waits for them.  The compiler fetches arguments where they are first
// used, behind branches, which at the start of a kernel costs one cold scalar-cache miss (about
// 0.3 us) after the other; with every line requested up front there is one such wait and the
// compiler's own loads hit.  The loaded words are not used.  The wait is part of the same asm
// statement on purpose: a scalar load writes its destination when the data returns, so the
// destination registers must stay reserved until then.
template <int BYTES> __device__ __forceinline__ void touch_kernargs() {
    static_assert(BYTES > 0 && BYTES <= 256, "one load per 64-byte line, four lines at most");
    const auto* ka = (const __attribute__((address_space(4))) uint32_t*)__builtin_amdgcn_kernarg_segment_ptr();
    uint32_t d0, d1, d2, d3;
    if (BYTES <= 64)
        asm volatile("s_load_dword %0, %1, 0x0\n\ts_waitcnt lgkmcnt(0)" : "=&s"(d0) : "s"(ka));
    else if (BYTES <= 128)
        asm volatile("s_load_dword %0, %2, 0x0\n\ts_load_dword %1, %2, 0x40\n\ts_waitcnt lgkmcnt(0)" : "=&s"(d0), "=&s"(d1) : "s"(ka));
    else if (BYTES <= 192)
        asm volatile("s_load_dword %0, %3, 0x0\n\ts_load_dword %1, %3, 0x40\n\ts_load_dword %2, %3, 0x80\n\ts_waitcnt lgkmcnt(0)"
                     : "=&s"(d0), "=&s"(d1), "=&s"(d2) : "s"(ka));
    else
        asm volatile("s_load_dword %0, %4, 0x0\n\ts_load_dword %1, %4, 0x40\n\ts_load_dword %2, %4, 0x80\n\ts_load_dword %3, %4, 0xc0\n\t"
                     "s_waitcnt lgkmcnt(0)" : "=&s"(d0), "=&s"(d1), "=&s"(d2), "=&s"(d3) : "s"(ka));
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

// Cache policy of the output stores (the `aux` operand of the buffer-store builtins; bit 4 = sc1 on gfx94x/gfx950):
// write through at system scope.  y is written once and never read back by the kernel; stored with the default
// policy its lines stay dirty in the L2 of the storing XCD until the release at the end of the kernel writes them
// back all at once, which is what 1.5-2.5 us at the end of every launch of the write-heavy layers consisted of.
// Written through, they leave while the kernel still runs (measured: 3x3 64->64 layer -15 %, 1x1 256->512 -16 %,
// 7x7 first layer -12 %, strided 3x3 -7 %, dilated 3x3 -5 %, 7x7-map 3x3 -3 %; sc0, nt and their combinations with
// sc1 are no better, nt alone makes the first layer 14 % slower).  It pays only for stores that cover whole 128-byte
// lines per instruction, which the staged epilogues do: written through in 8-byte pieces per lane a plain copy runs
// at 2.5 instead of 5.8 TB/s, so the stores through plain pointers (odd filter counts, the lowering kernels, the copy
// probe) keep the default policy.
constexpr int kStoreYPolicy = 16;

// Four consecutive fp32 results (one 16-byte staging piece) to a buffer, converted to the output
// type; an offset at or past the end of the buffer drops the store.
template <typename O> __device__ __forceinline__ void store_piece(u32x4 v, rsrc_t rsrc, uint32_t off);
template <> __device__ __forceinline__ void store_piece<float>(u32x4 v, rsrc_t rsrc, uint32_t off) {
    __builtin_amdgcn_raw_buffer_store_b128(v, rsrc, (int)off, 0, kStoreYPolicy);
}
template <> __device__ __forceinline__ void store_piece<bf16_t>(u32x4 v, rsrc_t rsrc, uint32_t off) {
    typedef bf16_t bf16x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const floatx4 f = __builtin_bit_cast(floatx4, v);
    const bf16x4 h = {to_out<bf16_t>(f[0]), to_out<bf16_t>(f[1]), to_out<bf16_t>(f[2]), to_out<bf16_t>(f[3])};
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, h), rsrc, (int)off, 0, kStoreYPolicy);
}
template <> __device__ __forceinline__ void store_piece<f16_t>(u32x4 v, rsrc_t rsrc, uint32_t off) {
    typedef f16_t f16x4 __attribute__((ext_vector_type(4)));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const floatx4 f = __builtin_bit_cast(floatx4, v);
    const f16x4 h = {(f16_t)f[0], (f16_t)f[1], (f16_t)f[2], (f16_t)f[3]};
    __builtin_amdgcn_raw_buffer_store_b64(__builtin_bit_cast(u32x2, h), rsrc, (int)off, 0, kStoreYPolicy);
}

// Bytes of wave-private LDS one call of store_frag_staged needs.
constexpr int kFragStageBytes = 2048;

// Output staging layout: byte offset of 16-byte piece `piece` (four filters, 0..7) of pixel `pixel` in a
// staging area of 128-byte pixel rows.  The deposit is a ds_write_b128 in which eight consecutive lanes
// hold the same piece of eight consecutive pixels, and the LDS serves a ds_write_b128 in passes of
// eight consecutive lanes that must hit eight different 16-byte slots modulo 128 bytes (measured with
// the bank-conflict counter on lane pairs): hence the xor with pixel % 8.  The read-back, lane l =
// piece l%8 of pixel l/8 (+8, +16, ..), is a ds_read_b128, served in passes of 16 lanes (see swz above)
// that must hit 16 different slots modulo 256 bytes; it does, two pixels x eight pieces per pass.
__host__ __device__ __forceinline__ constexpr uint32_t stage_off(int pixel, int piece) {
    return (uint32_t)(pixel * 128 + ((piece ^ (pixel & 7)) << 4));
}

// Writes one 32 x 32 accumulator fragment of the MFMA kernels to y through a wave-private LDS
// staging area, so that every store instruction covers whole 128-byte lines of y rows.  In the
// fragment lane l holds pixel l%32 and, in element v, filter 8*(v/4) + 4*(l/32) + v%4; written
// directly, one store instruction would touch 32 rows with 32 bytes each.  Half a fragment (16
// pixels x 32 filters, 2 KiB) goes through the staging area at a time: piece c (16 bytes, four
// filters) of pixel i sits at stage_off(i, c), which keeps both the deposit (16 pixels x 2 pieces per
// instruction) and the row-wise read-back free of bank conflicts.  The
// read-back gives lane l piece l%8 of pixels l/8 and l/8 + 8 of the half: eight lanes = one line.
// `row_off(i)` returns the byte offset, within the buffer of `y_rsrc`, of the first of the
// fragment's 32 filters in the y row of fragment pixel i, or an offset that the piece offset
// cannot bring back into range (e.g. 0x80000000 with fewer than 2^31 bytes in the buffer) to drop
// the pixel.  `pieces_ok` says whether this lane's four filters (piece l%8) exist.  `stg` is the
// wave's own staging area; LDS operations of one wave complete in order, so no wait is needed
// between the halves.
template <typename TO, typename RowOff>
__device__ __forceinline__ void store_frag_staged(char* stg, const floatx16& acc, int lane, rsrc_t y_rsrc, bool pieces_ok,
                                                  RowOff row_off) {
    const int frow = lane & 31, fk = lane >> 5, f16 = frow & 15;
    const int l8 = lane >> 3, c8 = lane & 7;
    const uint32_t sw0 = stage_off(f16, fk);         // piece 2*gq + fk: xor (gq << 5)
    const uint32_t sr0 = stage_off(l8, c8);
    const uint32_t sr1 = stage_off(l8 + 8, c8);
    u32x4 out[2][2];
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        __builtin_amdgcn_wave_barrier();
        if ((frow >> 4) == h) {
#pragma unroll
            for (int gq = 0; gq < 4; ++gq) {
                floatx4 v = {acc[4 * gq], acc[4 * gq + 1], acc[4 * gq + 2], acc[4 * gq + 3]};
                *reinterpret_cast<floatx4*>(stg + (sw0 ^ (uint32_t)(gq << 5))) = v;
            }
        }
        __builtin_amdgcn_wave_barrier();
        out[h][0] = *reinterpret_cast<const u32x4*>(stg + sr0);
        out[h][1] = *reinterpret_cast<const u32x4*>(stg + sr1);
    }
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const uint32_t ro = row_off(h * 16 + 8 * j + l8);
            if (pieces_ok) store_piece<TO>(out[h][j], y_rsrc, ro + (uint32_t)(4 * c8) * (uint32_t)sizeof(TO));
        }
}

}  // namespace iconv

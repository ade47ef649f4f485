// Shared declarations of the iconv HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "iconv.h"

namespace iconv {

// Problem description handed to every kernel by value.  Notation as in iconv.h.
struct ConvShape {
    int N, H, W, C, K, R, S;
    int stride, pad, dil;
    int P, Q;
    int M;       // N*P*Q   rows of the equivalent GEMM
    int PQ;      // P*Q
    int Kg;      // C*R*S   reduction length of the equivalent GEMM
};

typedef __bf16 bf16_t;
typedef _Float16 f16_t;

typedef bf16_t bf16x8 __attribute__((ext_vector_type(8)));
typedef f16_t f16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Element-type traits: storage type, MFMA fragment type and the 32x32x16 instruction.
template <typename T> struct Elem;
template <> struct Elem<bf16_t> {
    typedef bf16x8 frag;
    static __device__ __forceinline__ floatx16 mfma32(frag a, frag b, floatx16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
    }
};
template <> struct Elem<f16_t> {
    typedef f16x8 frag;
    static __device__ __forceinline__ floatx16 mfma32(frag a, frag b, floatx16 c) {
        return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
    }
};

// fp32 -> output element, round to nearest even.
template <typename O> __device__ __forceinline__ O to_out(float v);
template <> __device__ __forceinline__ float to_out<float>(float v) { return v; }
template <> __device__ __forceinline__ f16_t to_out<f16_t>(float v) { return (f16_t)v; }
// (gfx950 converts in hardware: v_cvt_pk_bf16_f32, round to nearest even, NaN stays NaN)
template <> __device__ __forceinline__ bf16_t to_out<bf16_t>(float v) { return (bf16_t)v; }

// ---- launchers implemented in the kernel translation units ---------------------------------
// in/out element codes used by the launch tables
enum InType { IN_F32 = 0, IN_BF16 = 1, IN_F16 = 2 };
enum OutType { OUT_F32 = 0, OUT_BF16 = 1, OUT_F16 = 2 };

hipError_t launch_direct(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t,
                         hipStream_t stream);

int mfma_num_variants();
const char* mfma_variant_name(int v);
bool mfma_variant_accepts(const ConvShape& s, int v);   // entry v runs the layer itself (C % 8 == 0 assumed)
int mfma_default_variant(const ConvShape& s);   // kernel-table entry chosen without an override (C % 8 == 0 layers)
// Picks a tile variant (or uses `variant` when >= 0) and launches the implicit-GEMM kernel.
// Requires C % 8 == 0 and a 16-bit input type.
hipError_t launch_mfma(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t,
                       int variant, hipStream_t stream);

// Patch-reuse kernels (channel chunk outer, tap inner; input patch resident in LDS).  Table order:
enum PatchVariant { kP128x64, kP256x128, kP256x64, kP64x64, kP64x128, kP128x64Staged, kP256x128Pf, kP64x128Pf, kP64x128C128,
                    kP64x128C128K2, kNumPatch };
int patch_num_variants();
const char* patch_variant_name(int v);
bool patch_supported(const ConvShape& s, int v);
hipError_t launch_patch(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v,
                        hipStream_t stream);

// Resident-filter kernels (C % 32 == 0, K <= 64, K % 4 == 0, filters and input patch fit in LDS).
int resident_num_variants();
const char* resident_variant_name(int v);
bool resident_supported(const ConvShape& s, int v);
int resident_choose(const ConvShape& s);   // best variant or -1
hipError_t launch_resident(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v,
                           hipStream_t stream);

// Resident-filter kernels phased by filter row, one LDS row per pixel (C == 32 or 64); variants 0, 1 = 7, 8 fragments
// with four compute and four loader waves, 2, 3 = the same with all eight waves computing (one block per workgroup).
bool rowres_supported(const ConvShape& s, int v);
bool rowres_plan_cost(const ConvShape& s, int v, double* cost, long* blocks);
hipError_t launch_rowres(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v, hipStream_t stream);

// Pixel-resident kernel for 1x1 layers (C = 64, 128 or 256; K % 4 == 0): a workgroup keeps its pixels in LDS and
// streams the filters through two teams of compute waves; variant 0: the compute waves store, 1: store waves do.
bool pointwise_supported(const ConvShape& s);
int pointwise_choose(const ConvShape& s);       // the form measured fastest on such layers, or -1: a per-tap kernel is faster
int pointwise_num_variants();
const char* pointwise_variant_name(int v);
hipError_t launch_pointwise(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v, hipStream_t stream);

// Merged-tap kernel for C == 4 first layers (stride 2, dilation 1, even W, S + (pad & 1) <= 8).
// Two forms (0: four waves per workgroup that load, multiply and store; 1: eight compute and four store waves);
// v outside the table, or a form the layer does not fit, means the form stem_choose names.
bool stem_supported(const ConvShape& s);
int stem_num_variants();
const char* stem_variant_name(int v);
bool stem_variant_supported(const ConvShape& s, int v);
int stem_choose(const ConvShape& s);
hipError_t launch_stem(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int v,
                       hipStream_t stream);

// Channel-last comparison kernel: NCHW input, KCRS filters, lowered columns ordered channel, tap row, tap column.
hipError_t launch_channel_last(const void* x_nchw, const void* w_kcrs, void* y, const ConvShape& s, int in_t, int out_t,
                               hipStream_t stream);

// lowered matrix with rows of `pitch_elems` elements (>= Kg, zero tail); 16-bit filter rows copied to a padded pitch
hipError_t launch_im2col(const void* x, void* lowered, const ConvShape& s, int elt_bytes, int pitch_elems, hipStream_t stream);
hipError_t launch_pad_rows(const void* src, void* dst, int rows, int len, int pitch, hipStream_t stream);
hipError_t launch_copy(void* dst, const void* src, size_t bytes, hipStream_t stream, bool write_through);
constexpr int kMfmaProbeGroups = 1024;   // workgroups of the MFMA probe (four per compute unit)
hipError_t launch_mfma_probe(void* out, int iters, bool random_operands, hipStream_t stream);
constexpr int kLdsProbePatterns = 8;
hipError_t launch_lds_probe(void* out, int iters, int pattern, hipStream_t stream);   // same grid and `out` as the MFMA probe
int lds_swizzle(int chunks_per_row, int row, int chunk);
int lds_stage_offset(int pixel, int piece);                // stage_off evaluated on the host   // swz<4> or swz<8> evaluated on the host

}  // namespace iconv

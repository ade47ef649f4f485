// C ABI of the library: argument checking, path selection, launches.  See include/iconv.h.
#include <atomic>

#include <initializer_list>

#include "iconv_bench.h"
#include "iconv_common.h"
#include "iconv_host.h"

using namespace iconv;

namespace {

// Launch width asked for by the iconv_fwd_ex call that is running on this thread (0 = fill the
// device).  Set and restored inside that one call, so no call sees another's value.
thread_local int tl_max_workgroups = 0;

// Workspace of iconv_fwd_explicit_noalloc: part of the device image, one copy per GPU.  In host code
// the name below is only a handle for hipGetSymbolAddress; the device address it yields (different on
// every GPU) is what the kernels get.
static __device__ __align__(256) unsigned char scratch[ICONV_NOALLOC_WORKSPACE_BYTES];
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device (looked up once per device), or nullptr.
void* scratch_on_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // concurrent first calls store the same address
    return p;
}

int out_dim(int in, int filt, int stride, int pad, int dil) {
    long span = (long)in + 2L * pad - (long)dil * (filt - 1) - 1;
    if (span < 0) return 0;
    return (int)(span / stride) + 1;
}

bool dtype_types(int dtype, int* in_t, int* out_t) {
    switch (dtype) {
        case ICONV_F32_F32:   *in_t = IN_F32;  *out_t = OUT_F32;  return true;
        case ICONV_BF16_F32:  *in_t = IN_BF16; *out_t = OUT_F32;  return true;
        case ICONV_F16_F32:   *in_t = IN_F16;  *out_t = OUT_F32;  return true;
        case ICONV_BF16_BF16: *in_t = IN_BF16; *out_t = OUT_BF16; return true;
        case ICONV_F16_F16:   *in_t = IN_F16;  *out_t = OUT_F16;  return true;
        default: return false;
    }
}

int in_bytes(int in_t) { return in_t == IN_F32 ? 4 : 2; }

// Validates the shape arguments and fills `s`.  Returns an ICONV_* status.
int make_shape(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int dil, ConvShape* s) {
    if (N < 1 || H < 1 || W < 1 || C < 1 || K < 1 || R < 1 || S < 1) return ICONV_ERR_SHAPE;
    if (stride < 1 || dil < 1 || pad < 0) return ICONV_ERR_SHAPE;
    const int P = out_dim(H, R, stride, pad, dil), Q = out_dim(W, S, stride, pad, dil);
    if (P < 1 || Q < 1) return ICONV_ERR_SHAPE;
    // every tensor, and the padded coordinate space the kernels index, must stay below 2^31 elements; the
    // products are formed one factor at a time so that absurd arguments cannot overflow on the way
    const long long lim = 1LL << 31;
    auto fits = [](long long limit, std::initializer_list<long long> factors) {
        long long prod = 1;
        for (long long f : factors) {
            if (f <= 0 || prod > limit / f) return false;       // prod * f would reach the limit (or f is not a size)
            prod *= f;
        }
        return prod < limit;
    };
    if (!fits(lim, {N, H, W, C}) || !fits(lim, {K, R, S, C}) || !fits(lim, {N, P, Q, K})) return ICONV_ERR_UNSUPPORTED;
    if (!fits(lim * 4, {H + 2LL * pad + (long long)dil * R, W + 2LL * pad + (long long)dil * S, C})) return ICONV_ERR_UNSUPPORTED;
    s->N = N; s->H = H; s->W = W; s->C = C; s->K = K; s->R = R; s->S = S;
    s->stride = stride; s->pad = pad; s->dil = dil; s->P = P; s->Q = Q;
    s->PQ = P * Q; s->M = N * P * Q; s->Kg = C * R * S;
    return ICONV_OK;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

int status_of(hipError_t e) { return e == hipSuccess ? ICONV_OK : ICONV_ERR_LAUNCH; }

// The launchers report hipGetLastError() after their launch; an error some earlier, unrelated HIP
// call left on this thread must not be taken for theirs, so it is consumed first.
void drop_stale_error() { (void)hipGetLastError(); }

// Runs the convolution with the fastest kernel that accepts the shape (variant < 0), or with the
// kernel-table entry `variant` where that entry can run it.  The table: the MFMA kernels for channel counts
// that are multiples of eight, then the forms of the merged-tap kernel for four-channel layers.
int run_conv(const void* x, const void* w, void* y, const ConvShape& s, int in_t, int out_t, int variant, hipStream_t st) {
    drop_stale_error();
    if (in_t != IN_F32 && (s.C % 8) == 0)
        return status_of(launch_mfma(x, w, y, s, in_t, out_t, variant, st));
    if (in_t != IN_F32 && stem_supported(s))
        return status_of(launch_stem(x, w, y, s, in_t, out_t, variant - mfma_num_variants(), st));
    return status_of(launch_direct(x, w, y, s, in_t, out_t, st));
}

// Workspace layout of the explicit variant: the lowered matrix, M rows of `pitch` elements, and -- when Kg is not
// a multiple of eight 16-bit elements, so that the MFMA GEMM cannot read the caller's filter matrix as it is --
// a copy of the K x Kg filter matrix with rows of the same pitch behind it.
struct ExplicitLayout {
    int pitch;              // elements per lowered row: Kg, or Kg rounded up to a multiple of 8 (16-bit inputs)
    size_t lowered_bytes;   // M * pitch * element size, rounded up to 16 bytes
    size_t filter_bytes;    // K * pitch * element size when the filters are copied, else 0
    size_t total() const { return lowered_bytes + filter_bytes; }
};
ExplicitLayout explicit_layout(const ConvShape& s, int in_t) {
    ExplicitLayout L;
    const size_t e = (size_t)in_bytes(in_t);
    const bool pad = in_t != IN_F32 && (s.Kg & 7) != 0;
    L.pitch = pad ? (s.Kg + 7) & ~7 : s.Kg;
    L.lowered_bytes = ((size_t)s.M * (size_t)L.pitch * e + 15) & ~(size_t)15;
    L.filter_bytes = pad ? (size_t)s.K * (size_t)L.pitch * e : 0;
    return L;
}

// Shape, type and lowered-matrix size of the explicit variant.  Returns an ICONV_* status.
int explicit_shape(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int dil, int dtype, ConvShape* s,
                   int* in_t, int* out_t, size_t* need) {
    int rc = make_shape(N, H, W, C, K, R, S, stride, pad, dil, s);
    if (rc != ICONV_OK) return rc;
    if (!dtype_types(dtype, in_t, out_t)) return ICONV_ERR_UNSUPPORTED;
    if ((size_t)s->M * (size_t)(s->Kg + 7) >= (1ull << 31)) return ICONV_ERR_UNSUPPORTED;
    *need = explicit_layout(*s, *in_t).total();
    return ICONV_OK;
}

// Lowering kernel into `workspace`, then the GEMM: a 1x1 stride-1 convolution over the lowered
// matrix seen as a 1 x 1 x M image with `pitch` channels; the KRSC filter tensor already is the
// K x Kg filter matrix in the same (tap-row, tap-column, channel) column order (copied to the
// padded pitch when the lowered rows are padded).
int run_explicit(const void* x, const void* w, void* y, void* workspace, const ConvShape& s, int in_t, int out_t,
                 hipStream_t st) {
    drop_stale_error();
    const ExplicitLayout L = explicit_layout(s, in_t);
    if (launch_im2col(x, workspace, s, in_bytes(in_t), L.pitch, st) != hipSuccess) return ICONV_ERR_LAUNCH;
    const void* wg = w;
    if (L.filter_bytes) {
        void* wp = static_cast<char*>(workspace) + L.lowered_bytes;
        if (launch_pad_rows(w, wp, s.K, s.Kg, L.pitch, st) != hipSuccess) return ICONV_ERR_LAUNCH;
        wg = wp;
    }
    ConvShape g;
    g.N = 1; g.H = 1; g.W = s.M; g.C = L.pitch; g.K = s.K; g.R = 1; g.S = 1;
    g.stride = 1; g.pad = 0; g.dil = 1; g.P = 1; g.Q = s.M; g.PQ = s.M; g.M = s.M; g.Kg = L.pitch;
    return run_conv(workspace, wg, y, g, in_t, out_t, -1, st);
}

}  // namespace

int iconv::call_max_workgroups() { return tl_max_workgroups; }

extern "C" {

int iconv_out_shape(int H, int W, int R, int S, int stride, int pad, int dilation, int* P, int* Q) {
    if (!P || !Q) return ICONV_ERR_NULL;
    if (H < 1 || W < 1 || R < 1 || S < 1 || stride < 1 || dilation < 1 || pad < 0) return ICONV_ERR_SHAPE;
    const int p = out_dim(H, R, stride, pad, dilation), q = out_dim(W, S, stride, pad, dilation);
    if (p < 1 || q < 1) return ICONV_ERR_SHAPE;
    *P = p; *Q = q;
    return ICONV_OK;
}

int iconv_fwd(const void* x, const void* w, void* y, int N, int H, int W, int C, int K, int R, int S,
              int stride, int pad, int dilation, int dtype, void* stream) {
    if (!x || !w || !y) return ICONV_ERR_NULL;
    ConvShape s;
    int rc = make_shape(N, H, W, C, K, R, S, stride, pad, dilation, &s);
    if (rc != ICONV_OK) return rc;
    int in_t, out_t;
    if (!dtype_types(dtype, &in_t, &out_t)) return ICONV_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return ICONV_ERR_ALIGN;
    return run_conv(x, w, y, s, in_t, out_t, -1, (hipStream_t)stream);
}

int iconv_fwd_ex(const void* x, const void* w, void* y, int N, int H, int W, int C, int K, int R, int S,
                 int stride, int pad, int dilation, int dtype, int variant, int max_workgroups, void* stream) {
    if (!x || !w || !y) return ICONV_ERR_NULL;
    ConvShape s;
    int rc = make_shape(N, H, W, C, K, R, S, stride, pad, dilation, &s);
    if (rc != ICONV_OK) return rc;
    int in_t, out_t;
    if (!dtype_types(dtype, &in_t, &out_t)) return ICONV_ERR_UNSUPPORTED;
    if (variant < -1 || variant >= iconv_num_variants() || max_workgroups < 0) return ICONV_ERR_UNSUPPORTED;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return ICONV_ERR_ALIGN;
    const int saved = tl_max_workgroups;
    tl_max_workgroups = max_workgroups;
    rc = run_conv(x, w, y, s, in_t, out_t, variant, (hipStream_t)stream);
    tl_max_workgroups = saved;
    return rc;
}

int iconv_fwd_channel_last(const void* x_nchw, const void* w_kcrs, void* y, int N, int H, int W, int C, int K, int R, int S,
                           int stride, int pad, int dilation, int dtype, void* stream) {
    if (!x_nchw || !w_kcrs || !y) return ICONV_ERR_NULL;
    ConvShape s;
    int rc = make_shape(N, H, W, C, K, R, S, stride, pad, dilation, &s);
    if (rc != ICONV_OK) return rc;
    int in_t, out_t;
    if (!dtype_types(dtype, &in_t, &out_t) || in_t == IN_F32) return ICONV_ERR_UNSUPPORTED;
    if (!aligned16(x_nchw) || !aligned16(w_kcrs) || !aligned16(y)) return ICONV_ERR_ALIGN;
    drop_stale_error();
    return status_of(launch_channel_last(x_nchw, w_kcrs, y, s, in_t, out_t, (hipStream_t)stream));
}

size_t iconv_workspace_bytes(int algo, int N, int H, int W, int C, int K, int R, int S, int stride, int pad,
                             int dilation, int dtype) {
    ConvShape s;
    int in_t, out_t;
    if (algo != ICONV_ALGO_EXPLICIT) return 0;
    if (make_shape(N, H, W, C, K, R, S, stride, pad, dilation, &s) != ICONV_OK) return 0;
    if (!dtype_types(dtype, &in_t, &out_t)) return 0;
    if ((size_t)s.M * (size_t)(s.Kg + 7) >= (1ull << 31)) return 0;
    return explicit_layout(s, in_t).total();
}

int iconv_im2col(const void* x, void* workspace, size_t workspace_bytes, int N, int H, int W, int C, int R, int S,
                 int stride, int pad, int dilation, int dtype, void* stream) {
    if (!x) return ICONV_ERR_NULL;
    ConvShape s;
    int rc = make_shape(N, H, W, C, 1, R, S, stride, pad, dilation, &s);
    if (rc != ICONV_OK) return rc;
    int in_t, out_t;
    if (!dtype_types(dtype, &in_t, &out_t)) return ICONV_ERR_UNSUPPORTED;
    if ((size_t)s.M * (size_t)(s.Kg + 7) >= (1ull << 31)) return ICONV_ERR_UNSUPPORTED;
    const ExplicitLayout L = explicit_layout(s, in_t);
    if (!workspace || workspace_bytes < L.lowered_bytes) return ICONV_ERR_WORKSPACE;
    if (!aligned16(x) || !aligned16(workspace)) return ICONV_ERR_ALIGN;
    drop_stale_error();
    return status_of(launch_im2col(x, workspace, s, in_bytes(in_t), L.pitch, (hipStream_t)stream));
}

int iconv_fwd_explicit(const void* x, const void* w, void* y, void* workspace, size_t workspace_bytes, int N, int H,
                       int W, int C, int K, int R, int S, int stride, int pad, int dilation, int dtype,
                       void* stream) {
    if (!x || !w || !y) return ICONV_ERR_NULL;
    ConvShape s;
    int in_t, out_t;
    size_t need = 0;
    int rc = explicit_shape(N, H, W, C, K, R, S, stride, pad, dilation, dtype, &s, &in_t, &out_t, &need);
    if (rc != ICONV_OK) return rc;
    if (!workspace || workspace_bytes < need) return ICONV_ERR_WORKSPACE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y) || !aligned16(workspace)) return ICONV_ERR_ALIGN;
    return run_explicit(x, w, y, workspace, s, in_t, out_t, (hipStream_t)stream);
}

int iconv_fwd_explicit_noalloc(const void* x, const void* w, void* y, int N, int H, int W, int C, int K, int R, int S,
                               int stride, int pad, int dilation, int dtype, void* stream) {
    if (!x || !w || !y) return ICONV_ERR_NULL;
    ConvShape s;
    int in_t, out_t;
    size_t need = 0;
    int rc = explicit_shape(N, H, W, C, K, R, S, stride, pad, dilation, dtype, &s, &in_t, &out_t, &need);
    if (rc != ICONV_OK) return rc;
    if (need > (size_t)ICONV_NOALLOC_WORKSPACE_BYTES) return ICONV_ERR_WORKSPACE;
    if (!aligned16(x) || !aligned16(w) || !aligned16(y)) return ICONV_ERR_ALIGN;
    void* ws = scratch_on_current_device();
    if (!ws) return ICONV_ERR_LAUNCH;
    return run_explicit(x, w, y, ws, s, in_t, out_t, (hipStream_t)stream);
}

int iconv_probe_copy(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return ICONV_ERR_NULL;
    if (bytes == 0 || (bytes & 15u)) return ICONV_ERR_SHAPE;
    if (!aligned16(dst) || !aligned16(src)) return ICONV_ERR_ALIGN;
    drop_stale_error();
    return status_of(launch_copy(dst, src, bytes, (hipStream_t)stream, false));
}

int iconv_probe_copy_wt(void* dst, const void* src, size_t bytes, void* stream) {
    if (!dst || !src) return ICONV_ERR_NULL;
    if (bytes == 0 || (bytes & 15u)) return ICONV_ERR_SHAPE;
    if (bytes >= (1ull << 32)) return ICONV_ERR_UNSUPPORTED;
    if (!aligned16(dst) || !aligned16(src)) return ICONV_ERR_ALIGN;
    drop_stale_error();
    return status_of(launch_copy(dst, src, bytes, (hipStream_t)stream, true));
}

int iconv_probe_mfma(void* out, size_t out_bytes, int iters, int random_operands, void* stream) {
    if (!out) return ICONV_ERR_NULL;
    if (iters < 1) return ICONV_ERR_SHAPE;
    if (out_bytes < (size_t)kMfmaProbeGroups * 256 * sizeof(float)) return ICONV_ERR_WORKSPACE;
    if (!aligned16(out)) return ICONV_ERR_ALIGN;
    drop_stale_error();
    return status_of(launch_mfma_probe(out, iters, random_operands != 0, (hipStream_t)stream));
}

int iconv_probe_lds(void* out, size_t out_bytes, int iters, int pattern, void* stream) {
    if (!out) return ICONV_ERR_NULL;
    if (iters < 1) return ICONV_ERR_SHAPE;
    if (pattern < 0 || pattern >= kLdsProbePatterns) return ICONV_ERR_UNSUPPORTED;
    if (out_bytes < (size_t)kMfmaProbeGroups * 256 * sizeof(float)) return ICONV_ERR_WORKSPACE;
    if (!aligned16(out)) return ICONV_ERR_ALIGN;
    drop_stale_error();
    return status_of(launch_lds_probe(out, iters, pattern, (hipStream_t)stream));
}

int iconv_lds_stage_offset(int pixel, int piece) {
    if (pixel < 0 || pixel >= (1 << 20) || piece < 0 || piece > 7) return -1;
    return lds_stage_offset(pixel, piece);
}

int iconv_lds_swizzle(int chunks_per_row, int row, int chunk) {
    if ((chunks_per_row != 4 && chunks_per_row != 8 && chunks_per_row != 16 && chunks_per_row != 32) || row < 0 || chunk < 0 ||
        chunk >= chunks_per_row)
        return -1;
    return lds_swizzle(chunks_per_row, row, chunk);
}

const char* iconv_kernel_for(int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int dilation, int dtype) {
    int in_t, out_t;
    ConvShape s;
    if (!dtype_types(dtype, &in_t, &out_t)) return nullptr;
    if (make_shape(N, H, W, C, K, R, S, stride, pad, dilation, &s) != ICONV_OK) return nullptr;
    // same order as run_conv
    if (in_t != IN_F32 && (s.C % 8) == 0) return mfma_variant_name(mfma_default_variant(s));
    if (in_t != IN_F32 && stem_supported(s)) return stem_variant_name(stem_choose(s));
    return "direct";
}

int iconv_num_variants(void) { return mfma_num_variants() + stem_num_variants(); }

int iconv_variant_accepts(int variant, int N, int H, int W, int C, int K, int R, int S, int stride, int pad, int dilation,
                          int dtype) {
    int in_t, out_t;
    ConvShape s;
    if (!dtype_types(dtype, &in_t, &out_t) || in_t == IN_F32) return 0;
    if (make_shape(N, H, W, C, K, R, S, stride, pad, dilation, &s) != ICONV_OK) return 0;
    if (variant >= mfma_num_variants()) return (s.C % 8) != 0 && stem_variant_supported(s, variant - mfma_num_variants()) ? 1 : 0;
    return (s.C % 8) == 0 && mfma_variant_accepts(s, variant) ? 1 : 0;
}

const char* iconv_variant_name(int variant) {
    if (variant < 0 || variant >= iconv_num_variants()) return "auto";
    if (variant >= mfma_num_variants()) return stem_variant_name(variant - mfma_num_variants());
    return mfma_variant_name(variant);
}

const char* iconv_status_string(int status) {
    switch (status) {
        case ICONV_OK: return "ok";
        case ICONV_ERR_NULL: return "null pointer";
        case ICONV_ERR_SHAPE: return "bad shape";
        case ICONV_ERR_UNSUPPORTED: return "unsupported dtype, algo or tensor size";
        case ICONV_ERR_ALIGN: return "pointer not 16-byte aligned";
        case ICONV_ERR_WORKSPACE: return "workspace missing or too small";
        case ICONV_ERR_LAUNCH: return "HIP launch failed";
        default: return "unknown status";
    }
}

}  // extern "C"

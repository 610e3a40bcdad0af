// Internal declarations shared by the HIP translation units of the library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include <atomic>

#include "snn.h"

namespace snn {

// Geometry of one layer as the kernels see it.
struct Geom {
    int N, C_in, C_out, H, W, stride, K;
    int Ho, Wo;          // output height and width
    int HoWo;            // Ho * Wo
    int64_t P;           // N * Ho * Wo output pixels
    int WW;              // words per packed row  (rows layout)
    int CW;              // words per packed pixel (channels layout)
};

inline Geom make_geom(const snn_conv_desc &d)
{
    Geom g;
    g.N = d.N; g.C_in = d.C_in; g.C_out = d.C_out; g.H = d.H; g.W = d.W;
    g.stride = d.stride; g.K = d.K;
    g.Ho = (d.H - 1) / d.stride + 1;
    g.Wo = (d.W - 1) / d.stride + 1;
    g.HoWo = g.Ho * g.Wo;
    g.P = (int64_t)d.N * g.HoWo;
    g.WW = (d.W + 31) / 32;
    g.CW = (d.C_in + 31) / 32;
    return g;
}

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Value of a tuning knob (SNN_TUNE_*): SNN_TUNE_AUTO unless set through snn_set_tuning or, once, from the environment.
int tuning(int knob);

// Border type of an output pixel: which rows / columns of its 3x3 window lie outside the image.
//   bit 0: top row, bit 1: bottom row, bit 2: left column, bit 3: right column.
__host__ __device__ inline int border_type(int ho, int wo, int H, int W, int stride)
{
    const int hc = ho * stride, wc = wo * stride;
    return (hc == 0 ? 1 : 0) | (hc + 1 >= H ? 2 : 0) | (wc == 0 ? 4 : 0) | (wc + 1 >= W ? 8 : 0);
}

__host__ __device__ inline int border_valid_taps(int type)
{
    return (3 - (type & 1) - ((type >> 1) & 1)) * (3 - ((type >> 2) & 1) - ((type >> 3) & 1));
}

// Window mask of the taps that lie outside the image, in "window order": bit (3*dy + dx).
__host__ __device__ inline uint32_t border_invalid_window(int type)
{
    uint32_t m = 0;
    if (type & 1) m |= 0x007u;   // dy = 0
    if (type & 2) m |= 0x1C0u;   // dy = 2
    if (type & 4) m |= 0x049u;   // dx = 0
    if (type & 8) m |= 0x124u;   // dx = 2
    return m;
}

// A 9-bit kernel code has tap t at bit (8 - t); kernels work on windows with tap t at bit t.
__host__ __device__ inline uint32_t code_to_window_order(uint32_t code)
{
    uint32_t r = 0;
    for (int t = 0; t < 9; ++t)
        r |= ((code >> (8 - t)) & 1u) << t;
    return r;
}

// ---- launchers (each validates nothing: the C entry points did) -----------------------------

int launch_pack_rows(const float *x, uint32_t *out, int64_t rows, int W, hipStream_t s);
int launch_pack_channels(const float *x, uint32_t *out, int N, int C, int H, int W, hipStream_t s);
// several tensors -> packed rows in one launch per group of 32 tensors
int launch_pack_rows_many(int n, const float *const *x, uint32_t *const *out, const int64_t *rows, const int *W, hipStream_t s);

int launch_project(const float *w, int64_t n, const uint16_t *codebook, int K, uint16_t *idx_out,
                   hipStream_t s);
int launch_project8(const float *w, int64_t n, const uint16_t *codebook8, int K, uint16_t *idx_out, hipStream_t s);

// A convolution is a small preparation kernel (weights -> tables in the workspace) and the
// convolution proper; callers whose weights stay fixed run the two separately.
enum : int { SNN_PHASE_PREPARE = 1, SNN_PHASE_CONVOLVE = 2, SNN_PHASE_BOTH = 3 };

size_t bnn_workspace_bytes(const Geom &g, int act);
int launch_bnn(const Geom &g, int act, const void *x, const uint16_t *w9, const float *alpha,
               float *y, void *ws, hipStream_t s, int phases = SNN_PHASE_BOTH);

// the same 1-bit layer as a dense FP4 contraction on the matrix cores (+-1 activations, packed channels)
bool dense_fp4_supported(const Geom &g);
size_t dense_fp4_workspace_bytes(const Geom &g);
// codebook == nullptr: `codes` are 9-bit kernel codes; else indices into the codebook (a sub-bit layer)
// sign_out != nullptr: instead of y, the next layer's packed channels, bit = ((float)S * alpha[co] + beta[co] >= 0),
// uint32 [N][H_out][W_out][ceil(C_out / 32)]
int launch_dense_fp4(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *codes, const float *alpha,
                     float *y, void *ws, hipStream_t s, int phases, const float *beta = nullptr,
                     uint32_t *sign_out = nullptr);

size_t subbit_workspace_bytes(const Geom &g, int act);
// one-hot slots per input channel of the form a layer is launched in (0: no matrix instructions)
int subbit_slots_per_channel(const Geom &g, int act);
int subbit_mfma_slots_per_channel(const Geom &g);
int launch_subbit(const Geom &g, int act, const void *x, const uint16_t *codebook,
                  const uint16_t *idx, const float *alpha, float *y, void *ws, hipStream_t s,
                  int phases = SNN_PHASE_BOTH);

// Optional ending of the sub-bit convolution: instead of y, the next layer's packed rows
// bit = ((float)S * alpha[co] + beta[co] >= 0), uint32 [N][C_out][H_out][ceil(W_out / 32)].
struct SignEpilogue {
    const float *beta;
    uint32_t *out;
};

// matrix-core variant of the sub-bit convolution (+-1 activations, K <= 64)
bool subbit_mfma_supported(const Geom &g);
size_t subbit_mfma_workspace_bytes(const Geom &g);
int launch_subbit_mfma(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx,
                       const float *alpha, float *y, void *ws, hipStream_t s, const SignEpilogue *sign = nullptr,
                       int phases = SNN_PHASE_BOTH, int tau = 0);
// tau > 0: `idx` is a stream of tau-bit indices (see snn_pack_indices) instead of uint16
int launch_pack_indices(const uint16_t *idx, int64_t n, int tau, uint32_t *out, hipStream_t s);

int launch_subbit_forward_mfma(const Geom &g, const float *x, const float *w, const uint16_t *codebook,
                               const float *alpha, uint16_t *idx_out, float *y, uint32_t *xr, void *ws, hipStream_t s,
                               const SignEpilogue *sign = nullptr);

// the convolutions of several prepared layers (matrix-core kernel, +-1 activations in packed rows, fp32 output)
int launch_subbit_mfma_many(int n_layers, const Geom *gs, const void *const *x, float *const *y, void *const *ws, hipStream_t s);

// the same with resident workers (one wave each) that draw (layer, tile) items from a counter in the first
// layer's workspace; `supported` says whether every layer has a form that kernel holds (at most 16 layers)
bool subbit_stack_supported(int n_layers, const Geom *gs);
int launch_subbit_stack(int n_layers, const Geom *gs, const void *const *x, float *const *y, void *const *ws, hipStream_t s);

int launch_subbit_prepare_many(int n_layers, const Geom *gs, const float *const *w, const uint16_t *const *codebook,
                               const float *const *alpha, const float *const *beta, uint16_t *const *idx_out,
                               void *const *ws, hipStream_t s);

// the two calls that end in the sign epilogue (packed rows in, packed rows out); UNSUPPORTED where
// the matrix-core kernel does not apply
int launch_subbit_sign(const Geom &g, const void *x_packed, const uint16_t *codebook, const uint16_t *idx,
                       const float *alpha, const float *beta, uint32_t *out_packed, void *ws, hipStream_t s,
                       int phases = SNN_PHASE_BOTH);
int launch_subbit_forward_sign(const Geom &g, const void *x_packed, const float *w, const uint16_t *codebook,
                               const float *alpha, const float *beta, uint16_t *idx_out, uint32_t *out_packed, void *ws,
                               hipStream_t s);

// Alg. 1 forward of one layer from fp32 activations and real-valued kernels (binary activations)
size_t subbit_forward_workspace_bytes(const Geom &g);
int launch_subbit_forward(const Geom &g, const float *x, const float *w, const uint16_t *codebook,
                          const float *alpha, uint16_t *idx_out, float *y, void *ws, hipStream_t s);

// Output activations are written once and not read again by the kernel that writes them: a
// non-temporal store lets them drain to memory while the kernel runs instead of waiting in L2 for
// the write-back at the kernel's end (measured: the kernels that follow run faster).
__device__ inline void store_output(float *p, float v) { __builtin_nontemporal_store(v, p); }

// fl(fl(a * b) + c): two fp32 roundings, never contracted into a fused multiply-add (the sign epilogue's
// definition; a threshold that sits exactly on an attained value must compare equal)
__device__ inline float mul_then_add(float a, float b, float c)
{
#pragma clang fp contract(off)
    const float prod = a * b;
    return prod + c;
}

// 1x1 layers: vectors of 8 input channels from a subset of {+-1}^8 (packed-channels input)
bool subbit_conv1x1_supported(const Geom &g);
size_t subbit_conv1x1_workspace_bytes(const Geom &g);
int launch_subbit_conv1x1(const Geom &g, const void *x, const uint16_t *codebook, const uint16_t *idx, const float *alpha,
                          float *y, void *ws, hipStream_t s, int phases = SNN_PHASE_BOTH);

// training side (Alg. 1 backward lines)
size_t project_backward_workspace_bytes(int64_t n, int K);
int launch_project_backward(const float *w, const float *g_wbar, const uint16_t *idx, int64_t n, int K, float *g_w,
                            float *g_p, void *ws, hipStream_t s);
int launch_subset_update(const float *p, int8_t *m, float theta, int K, uint16_t *codebook, uint8_t *dup, hipStream_t s);

// A kernel that asks for more than 64 KB of dynamic LDS needs its limit raised first: once per kernel, device
// and size (a launcher keeps one LdsGrant per kernel instantiation).
struct LdsGrant {
    static constexpr int MAX_DEVICES = 64;
    std::atomic<size_t> bytes[MAX_DEVICES];
};

inline int grant_dynamic_lds(const void *kernel, size_t lds, LdsGrant &grant)
{
    if (lds <= 64 * 1024) return SNN_OK;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return SNN_ERR_LAUNCH;
    const bool tracked = dev >= 0 && dev < LdsGrant::MAX_DEVICES;
    if (tracked && grant.bytes[dev].load(std::memory_order_acquire) >= lds) return SNN_OK;
    if (hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess) return SNN_ERR_LAUNCH;
    if (tracked) grant.bytes[dev].store(lds, std::memory_order_release);
    return SNN_OK;
}

inline int check_launch()
{
    return hipGetLastError() == hipSuccess ? SNN_OK : SNN_ERR_LAUNCH;
}

}  // namespace snn

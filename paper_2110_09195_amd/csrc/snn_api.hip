// C entry points of the library: argument checks, workspace sizing, dispatch.
#include "snn_internal.h"

#include <stdio.h>
#include <stdlib.h>

#include <atomic>
#include <mutex>
#include <vector>

using namespace snn;

// Scratch memory of snn_subbit_conv2d_noalloc: the convolution's workspace for callers that cannot
// allocate.  One copy per GPU the library runs on, held until the process ends.  In host code the
// name below is only a handle for hipGetSymbolAddress; the device address it returns is what the
// kernels receive.
static __device__ __align__(256) unsigned char scratch[SNN_NOALLOC_MAX_WORKSPACE_BYTES];

namespace {

constexpr int NOALLOC_MAX_DEVICES = 64;
void *g_scratch_ptr[NOALLOC_MAX_DEVICES];
std::mutex g_scratch_mutex;

// Device address of `scratch` on the current device (looked up once per device), or nullptr.
void *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= NOALLOC_MAX_DEVICES) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}

// ---- tuning knobs -----------------------------------------------------------------------------------------
std::atomic<int> g_tune[SNN_TUNE_COUNT];
std::once_flag g_tune_once;

bool tuning_value_ok(int knob, int v)
{
    if (v == SNN_TUNE_AUTO) return true;
    switch (knob) {
    case SNN_TUNE_MFMA_TILE: return v == 42 || v == 24 || v == 22 || v == 14 || v == 12;
    case SNN_TUNE_MFMA_KS: return v == 1 || v == 2 || v == 4;
    case SNN_TUNE_DENSE_TILE: return v >= 0 && v < 5;
    case SNN_TUNE_F32_WAVES: return v == 4 || v == 8 || v == 16;
    default: return v == 0 || v == 1;
    }
}

void tuning_from_environment()
{
    static const char *const names[SNN_TUNE_COUNT] = {"SNN_SUBBIT_MFMA", "SNN_MFMA_TILE", "SNN_MFMA_KS", "SNN_MFMA_STAGE",
                                                      "SNN_MFMA_QUAD",   "SNN_STACK",     "SNN_BNN_REGS", "SNN_DENSE_TILE",
                                                      "SNN_F32_WAVES"};
    for (int k = 0; k < SNN_TUNE_COUNT; ++k) {
        int v = SNN_TUNE_AUTO;
        if (const char *e = getenv(names[k])) {
            int a = 0, b = 0;
            if (k == SNN_TUNE_MFMA_TILE)
                v = sscanf(e, "%d,%d", &a, &b) == 2 ? 10 * a + b : SNN_TUNE_AUTO;
            else
                v = atoi(e);
            if (!tuning_value_ok(k, v)) v = SNN_TUNE_AUTO;
        }
        g_tune[k].store(v);
    }
}

bool desc_ok(const snn_conv_desc *d, bool need_K)
{
    if (!d) return false;
    if (d->N < 1 || d->C_in < 1 || d->C_out < 1 || d->H < 1 || d->W < 1) return false;
    if (d->C_in > 4096) return false;
    if (d->stride != 1 && d->stride != 2) return false;
    if (need_K && (d->K < 1 || d->K > 512)) return false;
    if (d->act != SNN_ACT_BIN_ROWS && d->act != SNN_ACT_BIN_CHANNELS && d->act != SNN_ACT_F32) return false;
    // element counts must fit the 32-bit pixel arithmetic of the kernels
    const int64_t in_elems = (int64_t)d->N * d->C_in * d->H * d->W;
    const int64_t out_elems = (int64_t)d->N * d->C_out * ((d->H - 1) / d->stride + 1) * ((d->W - 1) / d->stride + 1);
    if (in_elems >= ((int64_t)1 << 40) || out_elems >= ((int64_t)1 << 40)) return false;
    if ((int64_t)d->N * d->H * d->W >= ((int64_t)1 << 31)) return false;
    return true;
}

bool subbit_act_supported(int act) { return act == SNN_ACT_BIN_ROWS || act == SNN_ACT_F32; }

bool bnn_supported(const snn_conv_desc *d)
{
    return d->act == SNN_ACT_F32 || d->act == SNN_ACT_BIN_CHANNELS;
}

}  // namespace

int snn::tuning(int knob)
{
    std::call_once(g_tune_once, tuning_from_environment);
    return knob >= 0 && knob < SNN_TUNE_COUNT ? g_tune[knob].load(std::memory_order_relaxed) : SNN_TUNE_AUTO;
}

extern "C" {

int snn_set_tuning(int knob, int value)
{
    if (knob < 0 || knob >= SNN_TUNE_COUNT || !tuning_value_ok(knob, value)) return SNN_ERR_INVALID_ARG;
    std::call_once(g_tune_once, tuning_from_environment);
    g_tune[knob].store(value);
    return SNN_OK;
}

int snn_get_tuning(int knob) { return tuning(knob); }

int snn_subbit_slots_per_channel(const snn_conv_desc *desc)
{
    if (!desc_ok(desc, true)) return SNN_ERR_INVALID_ARG;
    return subbit_slots_per_channel(make_geom(*desc), desc->act);
}

const char *snn_status_string(int status)
{
    switch (status) {
    case SNN_OK: return "SNN_OK";
    case SNN_ERR_INVALID_ARG: return "SNN_ERR_INVALID_ARG";
    case SNN_ERR_UNSUPPORTED: return "SNN_ERR_UNSUPPORTED";
    case SNN_ERR_WORKSPACE: return "SNN_ERR_WORKSPACE";
    case SNN_ERR_LAUNCH: return "SNN_ERR_LAUNCH";
    default: return "SNN_ERR_UNKNOWN";
    }
}

size_t snn_packed_bytes(int N, int C, int H, int W, int layout)
{
    if (N < 1 || C < 1 || H < 1 || W < 1) return 0;
    switch (layout) {
    case SNN_ACT_BIN_ROWS: return (size_t)N * C * H * ((W + 31) / 32) * sizeof(uint32_t);
    case SNN_ACT_BIN_CHANNELS: return (size_t)N * H * W * ((C + 31) / 32) * sizeof(uint32_t);
    case SNN_ACT_F32: return (size_t)N * C * H * W * sizeof(float);
    default: return 0;
    }
}

size_t snn_workspace_bytes(const snn_conv_desc *desc, int which)
{
    if (which == SNN_WS_SUBBIT) {
        if (!desc_ok(desc, true) || !subbit_act_supported(desc->act)) return 0;
        return subbit_workspace_bytes(make_geom(*desc), desc->act);
    }
    if (which == SNN_WS_FORWARD) {
        if (!desc_ok(desc, true) || desc->act != SNN_ACT_BIN_ROWS) return 0;
        return subbit_forward_workspace_bytes(make_geom(*desc));
    }
    if (which == SNN_WS_CONV1X1) {
        if (!desc_ok(desc, true) || desc->act != SNN_ACT_BIN_CHANNELS) return 0;
        const Geom g = make_geom(*desc);
        return subbit_conv1x1_supported(g) ? subbit_conv1x1_workspace_bytes(g) : 0;
    }
    if (which == SNN_WS_BNN_DENSE) {
        if (!desc_ok(desc, false) || desc->act != SNN_ACT_BIN_CHANNELS) return 0;
        const Geom g = make_geom(*desc);
        return dense_fp4_supported(g) ? dense_fp4_workspace_bytes(g) : 0;
    }
    if (which == SNN_WS_BNN) {
        if (!desc_ok(desc, false) || !bnn_supported(desc)) return 0;
        return bnn_workspace_bytes(make_geom(*desc), desc->act);
    }
    return 0;
}

int snn_pack_activations(const float *x_nchw, void *packed, int N, int C, int H, int W, int layout,
                         void *stream)
{
    if (!x_nchw || !packed || N < 1 || C < 1 || H < 1 || W < 1) return SNN_ERR_INVALID_ARG;
    if ((int64_t)N * C * H * W >= ((int64_t)1 << 40) || (int64_t)H * W >= ((int64_t)1 << 31))
        return SNN_ERR_INVALID_ARG;
    hipStream_t s = (hipStream_t)stream;
    if (layout == SNN_ACT_BIN_ROWS)
        return launch_pack_rows(x_nchw, (uint32_t *)packed, (int64_t)N * C * H, W, s);
    if (layout == SNN_ACT_BIN_CHANNELS)
        return launch_pack_channels(x_nchw, (uint32_t *)packed, N, C, H, W, s);
    return SNN_ERR_INVALID_ARG;
}

int snn_pack_activations_many(const snn_pack_item *items, int n_items, void *stream)
{
    if (n_items < 0 || (n_items > 0 && !items)) return SNN_ERR_INVALID_ARG;
    std::vector<const float *> x;
    std::vector<uint32_t *> out;
    std::vector<int64_t> rows;
    std::vector<int> widths;
    for (int i = 0; i < n_items; ++i) {
        const snn_pack_item &it = items[i];
        if (!it.x_nchw || !it.packed || it.N < 1 || it.C < 1 || it.H < 1 || it.W < 1) return SNN_ERR_INVALID_ARG;
        if (it.layout != SNN_ACT_BIN_ROWS && it.layout != SNN_ACT_BIN_CHANNELS) return SNN_ERR_INVALID_ARG;
        if ((int64_t)it.N * it.C * it.H * it.W >= ((int64_t)1 << 40)) return SNN_ERR_INVALID_ARG;
    }
    for (int i = 0; i < n_items; ++i) {
        const snn_pack_item &it = items[i];
        if (it.layout == SNN_ACT_BIN_ROWS) {
            x.push_back(it.x_nchw);
            out.push_back((uint32_t *)it.packed);
            rows.push_back((int64_t)it.N * it.C * it.H);
            widths.push_back(it.W);
        } else {
            const int rc = launch_pack_channels(it.x_nchw, (uint32_t *)it.packed, it.N, it.C, it.H, it.W, (hipStream_t)stream);
            if (rc != SNN_OK) return rc;
        }
    }
    return launch_pack_rows_many((int)x.size(), x.data(), out.data(), rows.data(), widths.data(), (hipStream_t)stream);
}

int snn_project_kernels(const float *w, int64_t n, const uint16_t *codebook, int K, uint16_t *idx_out,
                        void *stream)
{
    if (n < 0 || K < 1 || K > 512 || !codebook) return SNN_ERR_INVALID_ARG;
    if (n == 0) return SNN_OK;
    if (!w || !idx_out) return SNN_ERR_INVALID_ARG;
    if (n >= ((int64_t)1 << 40)) return SNN_ERR_INVALID_ARG;
    return launch_project(w, n, codebook, K, idx_out, (hipStream_t)stream);
}

int snn_project_vectors8(const float *w, int64_t n, const uint16_t *codebook8, int K, uint16_t *idx_out,
                         void *stream)
{
    if (n < 0 || K < 1 || K > 256 || !codebook8) return SNN_ERR_INVALID_ARG;
    if (n == 0) return SNN_OK;
    if (!w || !idx_out || ((uintptr_t)w & 15u)) return SNN_ERR_INVALID_ARG;
    if (n >= ((int64_t)1 << 40)) return SNN_ERR_INVALID_ARG;
    return launch_project8(w, n, codebook8, K, idx_out, (hipStream_t)stream);
}

int snn_subbit_conv2d(const snn_conv_desc *desc, const void *x, const uint16_t *codebook,
                      const uint16_t *idx, const float *alpha, float *y_nchw, void *workspace,
                      size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !x || !codebook || !idx || !alpha || !y_nchw) return SNN_ERR_INVALID_ARG;
    if (!subbit_act_supported(desc->act)) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (need > 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u))) return SNN_ERR_WORKSPACE;
    return launch_subbit(g, desc->act, x, codebook, idx, alpha, y_nchw, workspace, (hipStream_t)stream);
}

int snn_subbit_conv2d_noalloc(const snn_conv_desc *desc, const void *x, const uint16_t *codebook, const uint16_t *idx,
                              const float *alpha, float *y_nchw, void *stream)
{
    if (!desc_ok(desc, true) || !x || !codebook || !idx || !alpha || !y_nchw) return SNN_ERR_INVALID_ARG;
    if (!subbit_act_supported(desc->act)) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (need > (size_t)SNN_NOALLOC_MAX_WORKSPACE_BYTES) return SNN_ERR_WORKSPACE;
    void *ws = scratch_on_current_device();
    if (!ws) return SNN_ERR_LAUNCH;
    return launch_subbit(g, desc->act, x, codebook, idx, alpha, y_nchw, ws, (hipStream_t)stream);
}

int snn_subbit_prepare(const snn_conv_desc *desc, const uint16_t *codebook, const uint16_t *idx, const float *alpha,
                       void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !codebook || !idx || !alpha) return SNN_ERR_INVALID_ARG;
    if (!subbit_act_supported(desc->act)) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (need > 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u))) return SNN_ERR_WORKSPACE;
    return launch_subbit(g, desc->act, nullptr, codebook, idx, alpha, nullptr, workspace, (hipStream_t)stream, SNN_PHASE_PREPARE);
}

size_t snn_packed_index_bytes(int64_t n, int tau)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || tau < 1 || tau > 9) return 0;
    return (size_t)((n * tau + 31) / 32) * sizeof(uint32_t);
}

int snn_pack_indices(const uint16_t *idx, int64_t n, int tau, void *packed, void *stream)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || tau < 1 || tau > 9) return SNN_ERR_INVALID_ARG;
    if (n == 0) return SNN_OK;
    if (!idx || !packed) return SNN_ERR_INVALID_ARG;
    return launch_pack_indices(idx, n, tau, (uint32_t *)packed, (hipStream_t)stream);
}

int snn_subbit_prepare_packed(const snn_conv_desc *desc, const uint16_t *codebook, const void *idx_packed, int tau,
                              const float *alpha, void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !codebook || !idx_packed || !alpha || tau < 1 || tau > 9) return SNN_ERR_INVALID_ARG;
    if (desc->K > (1 << tau)) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    if (!subbit_mfma_supported(g)) return SNN_ERR_UNSUPPORTED;
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_mfma(g, nullptr, codebook, (const uint16_t *)idx_packed, alpha, nullptr, workspace,
                              (hipStream_t)stream, nullptr, SNN_PHASE_PREPARE, tau);
}

int snn_subbit_conv2d_prepared(const snn_conv_desc *desc, const void *x, const float *alpha, float *y_nchw,
                               void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !x || !alpha || !y_nchw) return SNN_ERR_INVALID_ARG;
    if (!subbit_act_supported(desc->act)) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (need > 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u))) return SNN_ERR_WORKSPACE;
    return launch_subbit(g, desc->act, x, nullptr, nullptr, alpha, y_nchw, workspace, (hipStream_t)stream, SNN_PHASE_CONVOLVE);
}

int snn_subbit_forward(const snn_conv_desc *desc, const float *x_nchw, const float *w, const uint16_t *codebook,
                       const float *alpha, uint16_t *idx_out, float *y_nchw, void *workspace, size_t ws_bytes,
                       void *stream)
{
    if (!desc_ok(desc, true) || !x_nchw || !w || !codebook || !alpha || !idx_out || !y_nchw) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_forward_workspace_bytes(g);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_forward(g, x_nchw, w, codebook, alpha, idx_out, y_nchw, workspace, (hipStream_t)stream);
}

int snn_subbit_conv2d_sign(const snn_conv_desc *desc, const void *x_packed, const uint16_t *codebook,
                           const uint16_t *idx, const float *alpha, const float *beta, void *out_packed,
                           void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !x_packed || !codebook || !idx || !alpha || !beta || !out_packed) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_sign(g, x_packed, codebook, idx, alpha, beta, (uint32_t *)out_packed, workspace, (hipStream_t)stream);
}

int snn_subbit_prepare_sign(const snn_conv_desc *desc, const uint16_t *codebook, const uint16_t *idx,
                            const float *alpha, const float *beta, void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !codebook || !idx || !alpha || !beta) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_sign(g, nullptr, codebook, idx, alpha, beta, nullptr, workspace, (hipStream_t)stream, SNN_PHASE_PREPARE);
}

int snn_subbit_conv2d_sign_prepared(const snn_conv_desc *desc, const void *x_packed, void *out_packed, void *workspace,
                                    size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !x_packed || !out_packed) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_sign(g, x_packed, nullptr, nullptr, nullptr, nullptr, (uint32_t *)out_packed, workspace,
                              (hipStream_t)stream, SNN_PHASE_CONVOLVE);
}

int snn_subbit_project_prepare_many(const snn_layer_weights *layers, int n_layers, void *stream)
{
    if (n_layers < 0 || (n_layers > 0 && !layers)) return SNN_ERR_INVALID_ARG;
    if (n_layers == 0) return SNN_OK;
    std::vector<Geom> gs(n_layers);
    std::vector<const float *> w(n_layers), alpha(n_layers), beta(n_layers);
    std::vector<const uint16_t *> cb(n_layers);
    std::vector<uint16_t *> idx(n_layers);
    std::vector<void *> ws(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        const snn_layer_weights &L = layers[l];
        if (!desc_ok(&L.desc, true) || !L.w || !L.codebook || !L.alpha || !L.idx_out) return SNN_ERR_INVALID_ARG;
        if (L.desc.act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
        gs[l] = make_geom(L.desc);
        if (!subbit_mfma_supported(gs[l])) return SNN_ERR_UNSUPPORTED;
        const size_t need = subbit_workspace_bytes(gs[l], SNN_ACT_BIN_ROWS);
        if (!L.workspace || L.ws_bytes < need || ((uintptr_t)L.workspace & 255u)) return SNN_ERR_WORKSPACE;
        w[l] = L.w;
        cb[l] = L.codebook;
        alpha[l] = L.alpha;
        beta[l] = L.beta;
        idx[l] = L.idx_out;
        ws[l] = L.workspace;
    }
    return launch_subbit_prepare_many(n_layers, gs.data(), w.data(), cb.data(), alpha.data(), beta.data(), idx.data(), ws.data(),
                                      (hipStream_t)stream);
}

int snn_subbit_conv2d_prepared_many(const snn_layer_io *layers, int n_layers, void *stream)
{
    if (n_layers < 0 || (n_layers > 0 && !layers)) return SNN_ERR_INVALID_ARG;
    if (n_layers == 0) return SNN_OK;
    std::vector<Geom> gs(n_layers);
    std::vector<const void *> x(n_layers);
    std::vector<float *> y(n_layers);
    std::vector<void *> ws(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        const snn_layer_io &L = layers[l];
        if (!desc_ok(&L.desc, true) || !L.x_packed || !L.y_nchw) return SNN_ERR_INVALID_ARG;
        if (L.desc.act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
        gs[l] = make_geom(L.desc);
        if (!subbit_mfma_supported(gs[l])) return SNN_ERR_UNSUPPORTED;
        const size_t need = subbit_workspace_bytes(gs[l], SNN_ACT_BIN_ROWS);
        if (!L.workspace || L.ws_bytes < need || ((uintptr_t)L.workspace & 255u)) return SNN_ERR_WORKSPACE;
        x[l] = L.x_packed;
        y[l] = L.y_nchw;
        ws[l] = L.workspace;
    }
    if (tuning(SNN_TUNE_STACK) != 0 && subbit_stack_supported(n_layers, gs.data()))
        return launch_subbit_stack(n_layers, gs.data(), x.data(), y.data(), ws.data(), (hipStream_t)stream);
    return launch_subbit_mfma_many(n_layers, gs.data(), x.data(), y.data(), ws.data(), (hipStream_t)stream);
}

int snn_subbit_forward_many(const snn_layer_forward *layers, int n_layers, void *stream)
{
    if (n_layers < 0 || (n_layers > 0 && !layers)) return SNN_ERR_INVALID_ARG;
    if (n_layers == 0) return SNN_OK;
    std::vector<Geom> gs(n_layers);
    std::vector<const float *> x(n_layers), w(n_layers), alpha(n_layers);
    std::vector<const uint16_t *> codebook(n_layers);
    std::vector<uint16_t *> idx_out(n_layers);
    std::vector<uint32_t *> xr(n_layers);
    std::vector<const void *> xp(n_layers);
    std::vector<float *> y(n_layers);
    std::vector<void *> ws(n_layers);
    for (int l = 0; l < n_layers; ++l) {
        const snn_layer_forward &L = layers[l];
        if (!desc_ok(&L.desc, true) || !L.x_nchw || !L.w || !L.codebook || !L.alpha || !L.idx_out || !L.y_nchw)
            return SNN_ERR_INVALID_ARG;
        if (L.desc.act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
        gs[l] = make_geom(L.desc);
        if (!subbit_mfma_supported(gs[l])) return SNN_ERR_UNSUPPORTED;
        const size_t need = subbit_forward_workspace_bytes(gs[l]);
        if (!L.workspace || L.ws_bytes < need || ((uintptr_t)L.workspace & 255u)) return SNN_ERR_WORKSPACE;
        x[l] = L.x_nchw;
        w[l] = L.w;
        alpha[l] = L.alpha;
        codebook[l] = L.codebook;
        idx_out[l] = L.idx_out;
        xr[l] = (uint32_t *)((char *)L.workspace + align_up(subbit_workspace_bytes(gs[l], SNN_ACT_BIN_ROWS), 256));
        xp[l] = xr[l];
        y[l] = L.y_nchw;
        ws[l] = L.workspace;
    }
    std::vector<int64_t> rows(n_layers);
    std::vector<int> widths(n_layers);
    std::vector<const float *> no_beta(n_layers, nullptr);
    for (int l = 0; l < n_layers; ++l) {
        rows[l] = (int64_t)gs[l].N * gs[l].C_in * gs[l].H;
        widths[l] = gs[l].W;
    }
    int rc = launch_pack_rows_many(n_layers, x.data(), xr.data(), rows.data(), widths.data(), (hipStream_t)stream);
    if (rc != SNN_OK) return rc;
    rc = launch_subbit_prepare_many(n_layers, gs.data(), w.data(), codebook.data(), alpha.data(), no_beta.data(), idx_out.data(),
                                    ws.data(), (hipStream_t)stream);
    if (rc != SNN_OK) return rc;
    if (tuning(SNN_TUNE_STACK) != 0 && subbit_stack_supported(n_layers, gs.data()))
        return launch_subbit_stack(n_layers, gs.data(), xp.data(), y.data(), ws.data(), (hipStream_t)stream);
    return launch_subbit_mfma_many(n_layers, gs.data(), xp.data(), y.data(), ws.data(), (hipStream_t)stream);
}

int snn_subbit_forward_sign(const snn_conv_desc *desc, const void *x_packed, const float *w, const uint16_t *codebook,
                            const float *alpha, const float *beta, uint16_t *idx_out, void *out_packed,
                            void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !x_packed || !w || !codebook || !alpha || !beta || !idx_out || !out_packed)
        return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_ROWS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = subbit_workspace_bytes(g, desc->act);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_forward_sign(g, x_packed, w, codebook, alpha, beta, idx_out, (uint32_t *)out_packed, workspace,
                                      (hipStream_t)stream);
}

size_t snn_project_backward_workspace_bytes(int64_t n, int K)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || K < 1 || K > 512) return 0;
    return project_backward_workspace_bytes(n, K);
}

int snn_project_backward(const float *w, const float *g_wbar, const uint16_t *idx, int64_t n, int K, float *g_w,
                         float *g_p, void *workspace, size_t ws_bytes, void *stream)
{
    if (n < 0 || n >= ((int64_t)1 << 40) || K < 1 || K > 512 || !g_p) return SNN_ERR_INVALID_ARG;
    if (n > 0 && (!w || !g_wbar || !idx || !g_w)) return SNN_ERR_INVALID_ARG;
    if (!workspace || ws_bytes < project_backward_workspace_bytes(n, K) || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_project_backward(w, g_wbar, idx, n, K, g_w, g_p, workspace, (hipStream_t)stream);
}

int snn_subset_update(const float *p, int8_t *m, float theta, int K, uint16_t *codebook_out, uint8_t *dup_out,
                      void *stream)
{
    if (!p || !m || !codebook_out || !dup_out || K < 1 || K > 512 || !(theta >= 0.0f)) return SNN_ERR_INVALID_ARG;
    return launch_subset_update(p, m, theta, K, codebook_out, dup_out, (hipStream_t)stream);
}

int snn_subbit_conv1x1(const snn_conv_desc *desc, const void *x, const uint16_t *codebook8, const uint16_t *idx,
                       const float *alpha, float *y_nchw, void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !x || !codebook8 || !idx || !alpha || !y_nchw || desc->K > 256) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_CHANNELS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    if (!subbit_conv1x1_supported(g)) return SNN_ERR_UNSUPPORTED;
    const size_t need = subbit_conv1x1_workspace_bytes(g);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_conv1x1(g, x, codebook8, idx, alpha, y_nchw, workspace, (hipStream_t)stream);
}

int snn_subbit_conv1x1_prepare(const snn_conv_desc *desc, const uint16_t *codebook8, const uint16_t *idx, const float *alpha,
                               void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, true) || !codebook8 || !idx || !alpha || desc->K > 256) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_CHANNELS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    if (!subbit_conv1x1_supported(g)) return SNN_ERR_UNSUPPORTED;
    const size_t need = subbit_conv1x1_workspace_bytes(g);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_conv1x1(g, nullptr, codebook8, idx, alpha, nullptr, workspace, (hipStream_t)stream, SNN_PHASE_PREPARE);
}

int snn_subbit_conv1x1_prepared(const snn_conv_desc *desc, const void *x, float *y_nchw, void *workspace, size_t ws_bytes,
                                void *stream)
{
    if (!desc_ok(desc, true) || !x || !y_nchw || desc->K > 256) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_CHANNELS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    if (!subbit_conv1x1_supported(g)) return SNN_ERR_UNSUPPORTED;
    const size_t need = subbit_conv1x1_workspace_bytes(g);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_subbit_conv1x1(g, x, nullptr, nullptr, nullptr, y_nchw, workspace, (hipStream_t)stream, SNN_PHASE_CONVOLVE);
}

int snn_bnn_conv2d(const snn_conv_desc *desc, const void *x, const uint16_t *w9, const float *alpha,
                   float *y_nchw, void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, false) || !x || !w9 || !alpha || !y_nchw) return SNN_ERR_INVALID_ARG;
    if (!bnn_supported(desc)) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = bnn_workspace_bytes(g, desc->act);
    if (need > 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u))) return SNN_ERR_WORKSPACE;
    return launch_bnn(g, desc->act, x, w9, alpha, y_nchw, workspace, (hipStream_t)stream);
}

int snn_bnn_prepare(const snn_conv_desc *desc, const uint16_t *w9, void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, false) || !w9) return SNN_ERR_INVALID_ARG;
    if (!bnn_supported(desc)) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = bnn_workspace_bytes(g, desc->act);
    if (need > 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u))) return SNN_ERR_WORKSPACE;
    return launch_bnn(g, desc->act, nullptr, w9, nullptr, nullptr, workspace, (hipStream_t)stream, SNN_PHASE_PREPARE);
}

int snn_bnn_conv2d_prepared(const snn_conv_desc *desc, const void *x, const float *alpha, float *y_nchw,
                            void *workspace, size_t ws_bytes, void *stream)
{
    if (!desc_ok(desc, false) || !x || !alpha || !y_nchw) return SNN_ERR_INVALID_ARG;
    if (!bnn_supported(desc)) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    const size_t need = bnn_workspace_bytes(g, desc->act);
    if (need > 0 && (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u))) return SNN_ERR_WORKSPACE;
    return launch_bnn(g, desc->act, x, nullptr, alpha, y_nchw, workspace, (hipStream_t)stream, SNN_PHASE_CONVOLVE);
}

namespace {
int dense_call(const snn_conv_desc *desc, bool subbit, const void *x, const uint16_t *codebook, const uint16_t *codes,
               const float *alpha, float *y, void *workspace, size_t ws_bytes, void *stream, int phases,
               const float *beta = nullptr, uint32_t *sign_out = nullptr)
{
    if (!desc_ok(desc, subbit)) return SNN_ERR_INVALID_ARG;
    if ((phases & SNN_PHASE_PREPARE) && (!codes || (subbit && !codebook))) return SNN_ERR_INVALID_ARG;
    if ((phases & SNN_PHASE_CONVOLVE) && (!x || !alpha || (!y && !(beta && sign_out)))) return SNN_ERR_INVALID_ARG;
    if (desc->act != SNN_ACT_BIN_CHANNELS) return SNN_ERR_UNSUPPORTED;
    const Geom g = make_geom(*desc);
    if (!dense_fp4_supported(g)) return SNN_ERR_UNSUPPORTED;
    const size_t need = dense_fp4_workspace_bytes(g);
    if (!workspace || ws_bytes < need || ((uintptr_t)workspace & 255u)) return SNN_ERR_WORKSPACE;
    return launch_dense_fp4(g, x, subbit ? codebook : nullptr, codes, alpha, y, workspace, (hipStream_t)stream, phases, beta,
                            sign_out);
}
}  // namespace

int snn_bnn_conv2d_dense(const snn_conv_desc *desc, const void *x, const uint16_t *w9, const float *alpha,
                         float *y_nchw, void *workspace, size_t ws_bytes, void *stream)
{
    return dense_call(desc, false, x, nullptr, w9, alpha, y_nchw, workspace, ws_bytes, stream, SNN_PHASE_BOTH);
}

int snn_subbit_conv2d_dense(const snn_conv_desc *desc, const void *x, const uint16_t *codebook, const uint16_t *idx,
                            const float *alpha, float *y_nchw, void *workspace, size_t ws_bytes, void *stream)
{
    return dense_call(desc, true, x, codebook, idx, alpha, y_nchw, workspace, ws_bytes, stream, SNN_PHASE_BOTH);
}

int snn_dense_prepare(const snn_conv_desc *desc, const uint16_t *codebook, const uint16_t *codes, void *workspace,
                      size_t ws_bytes, void *stream)
{
    return dense_call(desc, codebook != nullptr, nullptr, codebook, codes, nullptr, nullptr, workspace, ws_bytes, stream,
                      SNN_PHASE_PREPARE);
}

int snn_dense_conv2d_prepared(const snn_conv_desc *desc, const void *x, const float *alpha, float *y_nchw,
                              void *workspace, size_t ws_bytes, void *stream)
{
    return dense_call(desc, false, x, nullptr, nullptr, alpha, y_nchw, workspace, ws_bytes, stream, SNN_PHASE_CONVOLVE);
}

int snn_dense_conv2d_sign_prepared(const snn_conv_desc *desc, const void *x, const float *alpha, const float *beta,
                                   void *out_packed, void *workspace, size_t ws_bytes, void *stream)
{
    if (!beta || !out_packed) return SNN_ERR_INVALID_ARG;
    return dense_call(desc, false, x, nullptr, nullptr, alpha, nullptr, workspace, ws_bytes, stream, SNN_PHASE_CONVOLVE, beta,
                      (uint32_t *)out_packed);
}

}  // extern "C"

// Host side of the C ABI: argument validation, shape bookkeeping and kernel dispatch.
// Every check happens before the first launch, so an error never leaves work half enqueued.
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "common.h"

using namespace purine;

namespace {

int64_t numel(const purine_tensor* t) {
    int64_t n = 1;
    for (int i = 0; i < t->ndim; ++i) n *= t->dim[i];
    return n;
}

// elements of one image (all axes but the first)
int64_t image_elems(const purine_tensor* t) {
    int64_t n = 1;
    for (int i = 1; i < t->ndim; ++i) n *= t->dim[i];
    return n;
}
// elements between consecutive images: the dense distance unless the tensor is a channel-slice view
int64_t nstride_of(const purine_tensor* t) {
    return (t->ndim == 4 && t->nstride != 0) ? t->nstride : image_elems(t);
}
bool is_view(const purine_tensor* t) { return nstride_of(t) != image_elems(t); }
// elements from the first to one past the last element of the tensor
int64_t span_elems(const purine_tensor* t) { return (t->dim[0] - 1) * nstride_of(t) + image_elems(t); }

static bool is_float_dtype_(int d) { return d == PURINE_F32 || d == PURINE_BF16; }
// allow_view: the argument may be a channel-slice view (F32 or BF16, 4 axes)
int check_tensor(const purine_tensor* t, int ndim, bool allow_view = false) {
    if (!t) return PURINE_E_NULL;
    if (!t->data) return PURINE_E_NULL;
    if (t->ndim != ndim) return PURINE_E_SHAPE;
    if (t->dtype != PURINE_F32 && t->dtype != PURINE_BF16 && t->dtype != PURINE_I32) return PURINE_E_DTYPE;
    int64_t n = 1;
    for (int i = 0; i < ndim; ++i) {
        if (t->dim[i] < 1) return PURINE_E_SHAPE;
        if (t->dim[i] >= (1ll << 31)) return PURINE_E_SHAPE;
        n *= t->dim[i];
        if (n >= (1ll << 31)) return PURINE_E_SHAPE;
    }
    if (((uintptr_t)t->data) & 15u) return PURINE_E_LAYOUT;
    if (t->nstride != 0) {
        if (t->ndim != 4 || t->nstride < image_elems(t)) return PURINE_E_SHAPE;
        if (is_view(t)) {
            // images keep the 16-byte alignment of the vector loads and stores: 4 floats, 8 bfloat16
            const int64_t packet = t->dtype == PURINE_BF16 ? 7 : 3;
            if (!allow_view || !is_float_dtype_(t->dtype) || (t->nstride & packet)) return PURINE_E_LAYOUT;
            if (t->nstride >= (1ll << 31) || span_elems(t) >= (1ll << 31)) return PURINE_E_SHAPE;
        }
    }
    return PURINE_OK;
}

bool is_float_dtype(int d) { return d == PURINE_F32 || d == PURINE_BF16; }
size_t elem_bytes(int d) { return d == PURINE_BF16 ? 2 : 4; }

// Do the two tensors share a byte? Exact for dense tensors; for two views with the same distance
// between images the per-image ranges are compared modulo that distance (channel slices of one
// buffer); anything else falls back to the spans.
bool overlaps(const purine_tensor* a, const purine_tensor* b) {
    const uintptr_t a0 = (uintptr_t)a->data, a1 = a0 + (size_t)span_elems(a) * elem_bytes(a->dtype);
    const uintptr_t b0 = (uintptr_t)b->data, b1 = b0 + (size_t)span_elems(b) * elem_bytes(b->dtype);
    if (!(a0 < b1 && b0 < a1)) return false;
    const uint64_t sa = (uint64_t)nstride_of(a) * elem_bytes(a->dtype), sb = (uint64_t)nstride_of(b) * elem_bytes(b->dtype);
    if (is_view(a) && is_view(b) && sa == sb) {
        const uint64_t la = (uint64_t)image_elems(a) * elem_bytes(a->dtype), lb = (uint64_t)image_elems(b) * elem_bytes(b->dtype);
        const uint64_t d = a0 >= b0 ? (a0 - b0) % sa : (sa - (b0 - a0) % sa) % sa;   // (a0 - b0) mod s
        return d < lb || sa - d < la;
    }
    return true;
}

bool same_dims(const purine_tensor* a, const purine_tensor* b) {
    if (a->ndim != b->ndim) return false;
    for (int i = 0; i < a->ndim; ++i)
        if (a->dim[i] != b->dim[i]) return false;
    return true;
}

int check_desc(const purine_conv_desc* d) {
    if (!d) return PURINE_E_NULL;
    if (d->stride_h < 1 || d->stride_w < 1 || d->pad_h < 0 || d->pad_w < 0) return PURINE_E_ARG;
    return PURINE_OK;
}

int check_beta(float beta) { return (beta == 0.0f || beta == 1.0f) ? PURINE_OK : PURINE_E_ARG; }

// Fills g from (desc, x extents, w extents) and verifies y extents when given.
int make_geom(const purine_conv_desc* d, const int64_t* xd, const int64_t* wd, const int64_t* yd,
              ConvGeom* g) {
    int64_t out[4];
    int rc = purine_conv_out_shape(d, xd, wd, out);
    if (rc != PURINE_OK) return rc;
    if (yd)
        for (int i = 0; i < 4; ++i)
            if (yd[i] != out[i]) return PURINE_E_SHAPE;
    // every extent and every index product used by the kernels must fit a signed 32-bit int
    const int64_t lim = (1ll << 31) - 1;
    if (xd[0] * xd[1] * xd[2] * xd[3] > lim || out[0] * out[1] * out[2] * out[3] > lim ||
        wd[0] * wd[1] * wd[2] * wd[3] > lim)
        return PURINE_E_SHAPE;
    if (wd[2] > 0xffff || wd[3] > 0xffff) return PURINE_E_SHAPE;
    g->N = (int)xd[0]; g->C = (int)xd[1]; g->H = (int)xd[2]; g->W = (int)xd[3];
    g->K = (int)wd[0]; g->R = (int)wd[2]; g->S = (int)wd[3];
    g->P = (int)out[2]; g->Q = (int)out[3];
    g->sh = d->stride_h; g->sw = d->stride_w; g->ph = d->pad_h; g->pw = d->pad_w;
    g->x_ns = g->C * g->H * g->W;
    g->y_ns = g->K * g->P * g->Q;
    // padded coordinates (h + pad, p*stride) also travel in 32-bit ints
    if ((int64_t)g->H + 2ll * g->ph > lim / 4 || (int64_t)g->W + 2ll * g->pw > lim / 4) return PURINE_E_SHAPE;
    return PURINE_OK;
}

}  // namespace

namespace purine {
static thread_local hipError_t g_last_hip_error = hipSuccess;
int hip_status(hipError_t e) {
    if (e == hipSuccess) return PURINE_OK;
    g_last_hip_error = e;
    return PURINE_E_HIP;
}
static thread_local KernelProbe g_probe{nullptr, nullptr};
KernelProbe take_kernel_probe() {
    KernelProbe p = g_probe;
    g_probe = KernelProbe{nullptr, nullptr};
    return p;
}
}  // namespace purine

extern "C" {

const char* purine_last_hip_error(void) { return hipGetErrorName(purine::g_last_hip_error); }

void purine_set_kernel_probe(void* start_event, void* stop_event) {
    purine::g_probe = KernelProbe{(hipEvent_t)start_event, (hipEvent_t)stop_event};
}

const char* purine_status_string(int status) {
    switch (status) {
        case PURINE_OK: return "ok";
        case PURINE_E_NULL: return "null pointer";
        case PURINE_E_SHAPE: return "inconsistent, empty or too large shape";
        case PURINE_E_DTYPE: return "unsupported dtype";
        case PURINE_E_LAYOUT: return "misaligned pointer or illegal aliasing";
        case PURINE_E_WORKSPACE: return "workspace missing or too small";
        case PURINE_E_GRAPH: return "not a legal bi-graph";
        case PURINE_E_HIP: return "HIP runtime error";
        case PURINE_E_ARG: return "scalar argument out of range";
        case PURINE_E_STATIC_SCRATCH: return "needs more scratch than the library's static device array holds";
        default: return "unknown status";
    }
}

int purine_conv_out_shape(const purine_conv_desc* desc, const int64_t x_dim[4],
                          const int64_t w_dim[4], int64_t y_dim[4]) {
    if (!desc || !x_dim || !w_dim || !y_dim) return PURINE_E_NULL;
    int rc = check_desc(desc);
    if (rc != PURINE_OK) return rc;
    for (int i = 0; i < 4; ++i)
        if (x_dim[i] < 1 || w_dim[i] < 1 || x_dim[i] >= (1ll << 31) || w_dim[i] >= (1ll << 31))
            return PURINE_E_SHAPE;
    if (x_dim[1] != w_dim[1]) return PURINE_E_SHAPE;
    const int64_t eh = x_dim[2] + 2ll * desc->pad_h - w_dim[2];
    const int64_t ew = x_dim[3] + 2ll * desc->pad_w - w_dim[3];
    if (eh < 0 || ew < 0) return PURINE_E_SHAPE;
    y_dim[0] = x_dim[0];
    y_dim[1] = w_dim[0];
    y_dim[2] = eh / desc->stride_h + 1;
    y_dim[3] = ew / desc->stride_w + 1;
    return PURINE_OK;
}

size_t purine_conv_workspace_bytes(int pass, const purine_conv_desc* desc, const int64_t x_dim[4],
                                   const int64_t w_dim[4], int32_t dtype) {
    if (pass < PURINE_CONV_FWD || pass > PURINE_CONV_BWD_WEIGHT_BIAS) return 0;
    if (!desc || !x_dim || !w_dim || !is_float_dtype(dtype)) return 0;
    ConvGeom g;
    if (make_geom(desc, x_dim, w_dim, nullptr, &g) != PURINE_OK) return 0;
    if (pass == PURINE_CONV_BWD_WEIGHT) return plan_wgrad(g, dtype).ws_bytes;
    if (pass == PURINE_CONV_BWD_WEIGHT_BIAS) {
        const WgradPlan pl = plan_wgrad(g, dtype);
        return wgrad_db_offset(pl) + pl.db_ws_bytes;
    }
    return plan_conv_pix(g, pass == PURINE_CONV_BWD_DATA, dtype, false).ws_bytes;
}

size_t purine_bias_bwd_workspace_bytes(const int64_t dy_dim[4], int32_t dtype) {
    if (!dy_dim || !is_float_dtype(dtype)) return 0;
    for (int i = 0; i < 4; ++i)
        if (dy_dim[i] < 1 || dy_dim[i] >= (1ll << 31)) return 0;
    if (dy_dim[0] * dy_dim[1] * dy_dim[2] * dy_dim[3] >= (1ll << 31)) return 0;
    return plan_bias_bwd((int)dy_dim[0], (int)dy_dim[1], (int)(dy_dim[2] * dy_dim[3])).ws_bytes;
}

// The bf16 multi-tap kernels address their channels-blocked copy of the gathered tensor with
// 32-bit byte offsets (range-checked raw buffer loads): the copy has to stay below 2^31 bytes.
static bool blocked_copy_too_large(const PixPlan& plan) {
    return plan.blk_offset != 0 && plan.ws_bytes - plan.blk_offset >= 0x7fffffffull;
}

static int conv_fwd_impl(const purine_conv_desc* desc, const purine_tensor* x, const purine_tensor* w,
                         const purine_tensor* b, purine_tensor* y, int relu, void* ws, size_t ws_bytes,
                         void* hip_stream) {
    int rc;
    if ((rc = check_desc(desc)) || (rc = check_tensor(x, 4, true)) || (rc = check_tensor(w, 4)) ||
        (rc = check_tensor(y, 4, true)))
        return rc;
    if (!is_float_dtype(x->dtype) || w->dtype != x->dtype || y->dtype != x->dtype) return PURINE_E_DTYPE;
    ConvGeom g;
    if ((rc = make_geom(desc, x->dim, w->dim, y->dim, &g))) return rc;
    g.x_ns = (int)nstride_of(x);
    g.y_ns = (int)nstride_of(y);
    if (overlaps(y, x) || overlaps(y, w)) return PURINE_E_LAYOUT;
    PixEpilogue epi;
    if (b) {
        if ((rc = check_tensor(b, 1))) return rc;
        if (b->dtype != y->dtype) return PURINE_E_DTYPE;
        if (b->dim[0] != y->dim[1]) return PURINE_E_SHAPE;
        if (overlaps(b, y)) return PURINE_E_LAYOUT;
        epi.bias = b->data;
    }
    if (relu != 0 && relu != 1) return PURINE_E_ARG;
    epi.relu = relu;
    const PixPlan plan = plan_conv_pix(g, false, x->dtype, epi.bias || epi.relu);
    if (blocked_copy_too_large(plan)) return PURINE_E_SHAPE;
    if (plan.ws_bytes && (!ws || ws_bytes < plan.ws_bytes)) return PURINE_E_WORKSPACE;
    if (plan.ws_bytes && (((uintptr_t)ws) & 15u)) return PURINE_E_LAYOUT;
    hipError_t e = launch_conv_pix(x->dtype, g, plan, x->data, w->data, y->data, 0.0f, ws, epi,
                                   (hipStream_t)hip_stream);
    return hip_status(e);
}

int purine_conv_fwd(const purine_conv_desc* desc, const purine_tensor* x, const purine_tensor* w,
                    purine_tensor* y, void* ws, size_t ws_bytes, void* hip_stream) {
    return conv_fwd_impl(desc, x, w, nullptr, y, 0, ws, ws_bytes, hip_stream);
}

int purine_conv_fwd_bias_relu(const purine_conv_desc* desc, const purine_tensor* x,
                              const purine_tensor* w, const purine_tensor* b, purine_tensor* y,
                              int relu, void* ws, size_t ws_bytes, void* hip_stream) {
    return conv_fwd_impl(desc, x, w, b, y, relu, ws, ws_bytes, hip_stream);
}

static int conv_bwd_data_impl(const purine_conv_desc* desc, const purine_tensor* dy,
                              const purine_tensor* w, const purine_tensor* act, purine_tensor* dx,
                              float beta, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_desc(desc)) || (rc = check_tensor(dy, 4, true)) || (rc = check_tensor(w, 4)) ||
        (rc = check_tensor(dx, 4, true)) || (rc = check_beta(beta)))
        return rc;
    if (!is_float_dtype(dy->dtype) || w->dtype != dy->dtype || dx->dtype != dy->dtype) return PURINE_E_DTYPE;
    ConvGeom g;
    if ((rc = make_geom(desc, dx->dim, w->dim, dy->dim, &g))) return rc;
    g.x_ns = (int)nstride_of(dx);
    g.y_ns = (int)nstride_of(dy);
    if (overlaps(dx, dy) || overlaps(dx, w)) return PURINE_E_LAYOUT;
    PixEpilogue epi;
    if (act) {
        if ((rc = check_tensor(act, 4, true))) return rc;
        if (act->dtype != dx->dtype) return PURINE_E_DTYPE;
        if (!same_dims(act, dx)) return PURINE_E_SHAPE;
        if (nstride_of(act) != nstride_of(dx)) return PURINE_E_LAYOUT;   // one set of offsets serves both
        if (overlaps(act, dx)) return PURINE_E_LAYOUT;
        epi.mask = act->data;
    }
    const PixPlan plan = plan_conv_pix(g, true, dy->dtype, epi.mask != nullptr, beta != 0.0f);
    if (blocked_copy_too_large(plan)) return PURINE_E_SHAPE;
    if (plan.ws_bytes && (!ws || ws_bytes < plan.ws_bytes)) return PURINE_E_WORKSPACE;
    if (plan.ws_bytes && (((uintptr_t)ws) & 15u)) return PURINE_E_LAYOUT;
    hipError_t e = launch_conv_pix(dy->dtype, g, plan, dy->data, w->data, dx->data, beta, ws, epi,
                                   (hipStream_t)hip_stream);
    return hip_status(e);
}

int purine_conv_bwd_data(const purine_conv_desc* desc, const purine_tensor* dy,
                         const purine_tensor* w, purine_tensor* dx, float beta, void* ws,
                         size_t ws_bytes, void* hip_stream) {
    return conv_bwd_data_impl(desc, dy, w, nullptr, dx, beta, ws, ws_bytes, hip_stream);
}

int purine_conv_bwd_data_relu(const purine_conv_desc* desc, const purine_tensor* dy,
                              const purine_tensor* w, const purine_tensor* act, purine_tensor* dx,
                              float beta, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!act) return PURINE_E_NULL;
    return conv_bwd_data_impl(desc, dy, w, act, dx, beta, ws, ws_bytes, hip_stream);
}

namespace {
// Scratch of the entry point that allocates nothing: one array in the device image of this
// library, so every GPU that loads the library holds its own copy until the process ends. In host
// code the name `scratch` is only a handle for hipGetSymbolAddress: the address a kernel may use
// is looked up once per device (with that device current) and kept in g_scratch_ptr.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];
constexpr int kMaxDevices = 64;
void* g_scratch_ptr[kMaxDevices];
std::mutex g_scratch_mu;

int static_scratch_of_current_device(void** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return hip_status(e);
    if (dev < 0 || dev >= kMaxDevices) return PURINE_E_ARG;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return hip_status(e);
        if (!p) return hip_status(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return PURINE_OK;
}

// db == nullptr: ConvBwdWeight alone. static_ws: the partial sums go to this device's static
// scratch array instead of a caller workspace (ws and ws_bytes are ignored).
int conv_bwd_weight_impl(const purine_conv_desc* desc, const purine_tensor* x, const purine_tensor* dy,
                         purine_tensor* dw, purine_tensor* db, float beta, void* ws, size_t ws_bytes,
                         void* hip_stream, bool static_ws = false) {
    int rc;
    if ((rc = check_desc(desc)) || (rc = check_tensor(x, 4, true)) || (rc = check_tensor(dy, 4, true)) ||
        (rc = check_tensor(dw, 4)) || (db && (rc = check_tensor(db, 1))) || (rc = check_beta(beta)))
        return rc;
    if (!is_float_dtype(x->dtype) || dy->dtype != x->dtype || dw->dtype != PURINE_F32) return PURINE_E_DTYPE;
    if (db && db->dtype != PURINE_F32) return PURINE_E_DTYPE;
    ConvGeom g;
    if ((rc = make_geom(desc, x->dim, dw->dim, dy->dim, &g))) return rc;
    g.x_ns = (int)nstride_of(x);
    g.y_ns = (int)nstride_of(dy);
    if (db && db->dim[0] != dy->dim[1]) return PURINE_E_SHAPE;
    if (overlaps(dw, x) || overlaps(dw, dy)) return PURINE_E_LAYOUT;
    if (db && (overlaps(db, x) || overlaps(db, dy) || overlaps(db, dw))) return PURINE_E_LAYOUT;
    const WgradPlan plan = plan_wgrad(g, x->dtype);
    const size_t need = db ? wgrad_db_offset(plan) + plan.db_ws_bytes : plan.ws_bytes;
    if (static_ws) {
        if (need > kStaticScratchBytes) return PURINE_E_STATIC_SCRATCH;
        if ((rc = static_scratch_of_current_device(&ws))) return rc;
        ws_bytes = kStaticScratchBytes;
    }
    if (!ws || ws_bytes < need) return PURINE_E_WORKSPACE;
    if (((uintptr_t)ws) & 15u) return PURINE_E_LAYOUT;
    hipError_t e = launch_conv_wgrad(x->dtype, g, plan, x->data, dy->data, (float*)dw->data,
                                     db ? (float*)db->data : nullptr, beta, ws, (hipStream_t)hip_stream);
    return hip_status(e);
}
}  // namespace

int purine_conv_bwd_weight(const purine_conv_desc* desc, const purine_tensor* x,
                           const purine_tensor* dy, purine_tensor* dw, float beta, void* ws,
                           size_t ws_bytes, void* hip_stream) {
    return conv_bwd_weight_impl(desc, x, dy, dw, nullptr, beta, ws, ws_bytes, hip_stream);
}

size_t purine_static_scratch_bytes(void) { return kStaticScratchBytes; }

int purine_conv_bwd_weight_static(const purine_conv_desc* desc, const purine_tensor* x,
                                  const purine_tensor* dy, purine_tensor* dw, float beta,
                                  void* hip_stream) {
    return conv_bwd_weight_impl(desc, x, dy, dw, nullptr, beta, nullptr, 0, hip_stream, true);
}

int purine_conv_bwd_weight_bias(const purine_conv_desc* desc, const purine_tensor* x,
                                const purine_tensor* dy, purine_tensor* dw, purine_tensor* db,
                                float beta, void* ws, size_t ws_bytes, void* hip_stream) {
    if (!db) return PURINE_E_NULL;
    return conv_bwd_weight_impl(desc, x, dy, dw, db, beta, ws, ws_bytes, hip_stream);
}

int purine_bias_fwd(const purine_tensor* b, purine_tensor* y, void* hip_stream) {
    int rc;
    if ((rc = check_tensor(b, 1)) || (rc = check_tensor(y, 4))) return rc;
    if (!is_float_dtype(y->dtype) || b->dtype != y->dtype) return PURINE_E_DTYPE;
    if (b->dim[0] != y->dim[1]) return PURINE_E_SHAPE;
    if (overlaps(b, y)) return PURINE_E_LAYOUT;
    hipError_t e = launch_bias_fwd(y->dtype, b->data, y->data, (int)y->dim[0], (int)y->dim[1],
                                   (int)(y->dim[2] * y->dim[3]), (hipStream_t)hip_stream);
    return hip_status(e);
}

int purine_bias_bwd(const purine_tensor* dy, purine_tensor* db, float beta, void* ws,
                    size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_tensor(dy, 4)) || (rc = check_tensor(db, 1)) || (rc = check_beta(beta))) return rc;
    if (!is_float_dtype(dy->dtype) || db->dtype != PURINE_F32) return PURINE_E_DTYPE;
    if (db->dim[0] != dy->dim[1]) return PURINE_E_SHAPE;
    if (overlaps(db, dy)) return PURINE_E_LAYOUT;
    const int N = (int)dy->dim[0], K = (int)dy->dim[1], PQ = (int)(dy->dim[2] * dy->dim[3]);
    const BiasBwdPlan plan = plan_bias_bwd(N, K, PQ);
    if (!ws || ws_bytes < plan.ws_bytes) return PURINE_E_WORKSPACE;
    if (((uintptr_t)ws) & 15u) return PURINE_E_LAYOUT;
    hipError_t e = launch_bias_bwd(dy->dtype, dy->data, (float*)db->data, beta, N, K, PQ, plan, ws,
                                   (hipStream_t)hip_stream);
    return hip_status(e);
}

int purine_relu_fwd(const purine_tensor* x, purine_tensor* y, void* hip_stream) {
    int rc;
    if (!x || !y) return PURINE_E_NULL;
    if ((rc = check_tensor(x, x->ndim >= 1 && x->ndim <= 4 ? x->ndim : -1, true)) ||
        (rc = check_tensor(y, x->ndim, true)))
        return rc;
    if (!is_float_dtype(x->dtype) || y->dtype != x->dtype) return PURINE_E_DTYPE;
    if (!same_dims(x, y)) return PURINE_E_SHAPE;
    if (x->data == y->data ? nstride_of(x) != nstride_of(y) : overlaps(x, y)) return PURINE_E_LAYOUT;
    hipError_t e;
    if (is_view(x) || is_view(y)) {
        if (x->dim[0] > 65535) return PURINE_E_SHAPE;
        e = launch_relu_view(x->dtype, false, x->data, nullptr, y->data, (int)x->dim[0],
                             (int)image_elems(x), nstride_of(x), 0, nstride_of(y), (hipStream_t)hip_stream);
    } else {
        e = launch_relu_fwd(x->dtype, x->data, y->data, numel(x), (hipStream_t)hip_stream);
    }
    return hip_status(e);
}

int purine_relu_bwd(const purine_tensor* x, const purine_tensor* dy, purine_tensor* dx,
                    void* hip_stream) {
    int rc;
    if (!x || !dy || !dx) return PURINE_E_NULL;
    if ((rc = check_tensor(x, x->ndim >= 1 && x->ndim <= 4 ? x->ndim : -1, true)) ||
        (rc = check_tensor(dy, x->ndim, true)) || (rc = check_tensor(dx, x->ndim, true)))
        return rc;
    if (!is_float_dtype(x->dtype) || dy->dtype != x->dtype || dx->dtype != x->dtype) return PURINE_E_DTYPE;
    if (!same_dims(x, dy) || !same_dims(x, dx)) return PURINE_E_SHAPE;
    if (overlaps(dx, x)) return PURINE_E_LAYOUT;
    if (dx->data == dy->data ? nstride_of(dx) != nstride_of(dy) : overlaps(dx, dy)) return PURINE_E_LAYOUT;
    hipError_t e;
    if (is_view(x) || is_view(dy) || is_view(dx)) {
        if (x->dim[0] > 65535) return PURINE_E_SHAPE;
        e = launch_relu_view(x->dtype, true, x->data, dy->data, dx->data,
                             (int)x->dim[0], (int)image_elems(x), nstride_of(x), nstride_of(dy),
                             nstride_of(dx), (hipStream_t)hip_stream);
    } else {
        e = launch_relu_bwd(x->dtype, x->data, dy->data, dx->data, numel(x), (hipStream_t)hip_stream);
    }
    return hip_status(e);
}

int purine_sgd_update(const purine_tensor* w, const purine_tensor* dw, purine_tensor* new_w,
                      float lr, void* hip_stream) {
    int rc;
    if (!w || !dw || !new_w) return PURINE_E_NULL;
    if ((rc = check_tensor(w, w->ndim >= 1 && w->ndim <= 4 ? w->ndim : -1)) ||
        (rc = check_tensor(dw, w->ndim)) || (rc = check_tensor(new_w, w->ndim)))
        return rc;
    if (!is_float_dtype(w->dtype) || new_w->dtype != w->dtype || dw->dtype != PURINE_F32) return PURINE_E_DTYPE;
    if (!same_dims(w, dw) || !same_dims(w, new_w)) return PURINE_E_SHAPE;
    if (!(lr == lr) || lr - lr != 0.0f) return PURINE_E_ARG;   // NaN or infinite step
    if (new_w->data != w->data && overlaps(new_w, w)) return PURINE_E_LAYOUT;
    if (overlaps(new_w, dw)) return PURINE_E_LAYOUT;
    hipError_t e = launch_sgd_update(w->dtype, w->data, (const float*)dw->data, new_w->data, lr, numel(w),
                                     (hipStream_t)hip_stream);
    return hip_status(e);
}

static int pool_geom(const purine_pool_desc* d, const purine_tensor* x, const purine_tensor* y) {
    if (!d) return PURINE_E_NULL;
    if (d->window < 1 || d->stride < 1 || d->pad < 0 || d->pad >= d->window) return PURINE_E_ARG;
    for (int ax = 2; ax < 4; ++ax) {
        const int64_t e = x->dim[ax] + 2ll * d->pad - d->window;
        if (e < 0) return PURINE_E_SHAPE;
        if (y->dim[ax] != e / d->stride + 1) return PURINE_E_SHAPE;
    }
    if (y->dim[0] != x->dim[0] || y->dim[1] != x->dim[1]) return PURINE_E_SHAPE;
    if (x->dim[0] * x->dim[1] >= (1ll << 31)) return PURINE_E_SHAPE;
    return PURINE_OK;
}

int purine_maxpool_fwd(const purine_pool_desc* desc, const purine_tensor* x, purine_tensor* y,
                       purine_tensor* arg, void* hip_stream) {
    int rc;
    if ((rc = check_tensor(x, 4)) || (rc = check_tensor(y, 4)) || (rc = check_tensor(arg, 4))) return rc;
    if (!is_float_dtype(x->dtype) || y->dtype != x->dtype || arg->dtype != PURINE_I32) return PURINE_E_DTYPE;
    if ((rc = pool_geom(desc, x, y))) return rc;
    if (!same_dims(y, arg)) return PURINE_E_SHAPE;
    if (overlaps(y, x) || overlaps(arg, x) || overlaps(arg, y)) return PURINE_E_LAYOUT;
    hipError_t e = launch_maxpool_fwd(x->dtype, x->data, y->data, (int32_t*)arg->data,
                                      (int)(x->dim[0] * x->dim[1]), (int)x->dim[2], (int)x->dim[3],
                                      (int)y->dim[2], (int)y->dim[3], desc->window, desc->stride,
                                      desc->pad, (hipStream_t)hip_stream);
    return hip_status(e);
}

namespace {
int maxpool_bwd_impl(const purine_pool_desc* desc, const purine_tensor* dy, const purine_tensor* arg,
                     const purine_tensor* y, purine_tensor* dx, float beta, void* hip_stream) {
    int rc;
    if ((rc = check_tensor(dy, 4)) || (rc = check_tensor(arg, 4)) || (rc = check_tensor(dx, 4)) ||
        (y && (rc = check_tensor(y, 4))) || (rc = check_beta(beta)))
        return rc;
    if (!is_float_dtype(dy->dtype) || dx->dtype != dy->dtype || arg->dtype != PURINE_I32) return PURINE_E_DTYPE;
    if (y && y->dtype != dy->dtype) return PURINE_E_DTYPE;
    if ((rc = pool_geom(desc, dx, dy))) return rc;
    if (!same_dims(dy, arg) || (y && !same_dims(y, dy))) return PURINE_E_SHAPE;
    if (overlaps(dx, dy) || overlaps(dx, arg) || (y && overlaps(dx, y))) return PURINE_E_LAYOUT;
    hipError_t e = launch_maxpool_bwd(dy->dtype, dy->data, (const int32_t*)arg->data, dx->data,
                                      y ? y->data : nullptr, beta,
                                      (int)(dx->dim[0] * dx->dim[1]), (int)dx->dim[2],
                                      (int)dx->dim[3], (int)dy->dim[2], (int)dy->dim[3],
                                      desc->window, desc->stride, desc->pad, (hipStream_t)hip_stream);
    return hip_status(e);
}
}  // namespace

int purine_maxpool_bwd(const purine_pool_desc* desc, const purine_tensor* dy,
                       const purine_tensor* arg, purine_tensor* dx, float beta, void* hip_stream) {
    return maxpool_bwd_impl(desc, dy, arg, nullptr, dx, beta, hip_stream);
}

int purine_maxpool_bwd_relu(const purine_pool_desc* desc, const purine_tensor* dy, const purine_tensor* arg,
                            const purine_tensor* y, purine_tensor* dx, float beta, void* hip_stream) {
    if (!y) return PURINE_E_NULL;
    return maxpool_bwd_impl(desc, dy, arg, y, dx, beta, hip_stream);
}

static int concat_check(const purine_tensor* const* parts, int n_parts, const purine_tensor* whole) {
    if (!parts || !whole) return PURINE_E_NULL;
    if (n_parts < 1 || n_parts > 64) return PURINE_E_ARG;
    int rc = check_tensor(whole, 4);
    if (rc) return rc;
    if (!is_float_dtype(whole->dtype)) return PURINE_E_DTYPE;
    if (whole->dim[0] > 65535) return PURINE_E_SHAPE;
    int64_t c = 0;
    for (int i = 0; i < n_parts; ++i) {
        if ((rc = check_tensor(parts[i], 4))) return rc;
        if (parts[i]->dtype != whole->dtype) return PURINE_E_DTYPE;
        if (parts[i]->dim[0] != whole->dim[0] || parts[i]->dim[2] != whole->dim[2] ||
            parts[i]->dim[3] != whole->dim[3])
            return PURINE_E_SHAPE;
        if (overlaps(parts[i], whole)) return PURINE_E_LAYOUT;
        c += parts[i]->dim[1];
    }
    return c == whole->dim[1] ? PURINE_OK : PURINE_E_SHAPE;
}

int purine_concat_fwd(const purine_tensor* const* parts, int n_parts, purine_tensor* out,
                      void* hip_stream) {
    int rc = concat_check(parts, n_parts, out);
    if (rc) return rc;
    int c0 = 0;
    const int HW = (int)(out->dim[2] * out->dim[3]);
    for (int i = 0; i < n_parts; ++i) {
        const int c = (int)parts[i]->dim[1];
        hipError_t e = launch_copy_channels(out->dtype, parts[i]->data, out->data, (int)out->dim[0], c,
                                            c, 0, (int)out->dim[1], c0, HW, (hipStream_t)hip_stream);
        if (e != hipSuccess) return hip_status(e);
        c0 += c;
    }
    return PURINE_OK;
}

int purine_concat_bwd(const purine_tensor* dout, purine_tensor* const* dparts, int n_parts,
                      void* hip_stream) {
    int rc = concat_check((const purine_tensor* const*)dparts, n_parts, dout);
    if (rc) return rc;
    int c0 = 0;
    const int HW = (int)(dout->dim[2] * dout->dim[3]);
    for (int i = 0; i < n_parts; ++i) {
        const int c = (int)dparts[i]->dim[1];
        hipError_t e = launch_copy_channels(dout->dtype, dout->data, dparts[i]->data, (int)dout->dim[0],
                                            c, (int)dout->dim[1], c0, c, 0, HW, (hipStream_t)hip_stream);
        if (e != hipSuccess) return hip_status(e);
        c0 += c;
    }
    return PURINE_OK;
}

int purine_sum(const purine_tensor* const* terms, int n_terms, purine_tensor* out, void* hip_stream) {
    if (!terms || !out) return PURINE_E_NULL;
    if (n_terms < 1 || n_terms > 8) return PURINE_E_ARG;
    int rc;
    if (out->ndim < 1 || out->ndim > 4) return PURINE_E_SHAPE;
    if ((rc = check_tensor(out, out->ndim))) return rc;
    if (!is_float_dtype(out->dtype)) return PURINE_E_DTYPE;
    const void* ptrs[8];
    for (int i = 0; i < n_terms; ++i) {
        if ((rc = check_tensor(terms[i], out->ndim))) return rc;
        if (terms[i]->dtype != out->dtype) return PURINE_E_DTYPE;
        if (!same_dims(terms[i], out)) return PURINE_E_SHAPE;
        if (terms[i]->data != out->data && overlaps(terms[i], out)) return PURINE_E_LAYOUT;
        if (terms[i]->data == out->data && i != 0) return PURINE_E_LAYOUT;
        ptrs[i] = terms[i]->data;
    }
    hipError_t e = launch_sum(out->dtype, ptrs, n_terms, out->data, numel(out), (hipStream_t)hip_stream);
    return hip_status(e);
}

// ---- grouped convolution and fully-connected layer: compositions of the operators above -------

namespace {

// Channel slice [c0, c0 + count) of an NCHW tensor (dense or itself a view), as a view.
purine_tensor channel_slice(const purine_tensor* t, int64_t c0, int64_t count) {
    purine_tensor v = *t;
    v.data = (char*)t->data + (size_t)(c0 * t->dim[2] * t->dim[3]) * elem_bytes(t->dtype);
    v.dim[1] = count;
    v.nstride = nstride_of(t);
    return v;
}
// Rows [r0, r0 + count) of a dense tensor whose first axis is rows.
purine_tensor row_slice(const purine_tensor* t, int64_t r0, int64_t count) {
    purine_tensor v = *t;
    int64_t per_row = 1;
    for (int i = 1; i < t->ndim; ++i) per_row *= t->dim[i];
    v.data = (char*)t->data + (size_t)(r0 * per_row) * elem_bytes(t->dtype);
    v.dim[0] = count;
    return v;
}

// Everything a grouped call needs to know before its first launch: extents divide by the group
// count and every group's slices keep the alignment rules of views and dense tensors.
int check_groups(int groups, const purine_tensor* x, const purine_tensor* w, const purine_tensor* y) {
    int rc;
    if (groups < 1) return PURINE_E_ARG;
    if ((rc = check_tensor(x, 4, true)) || (rc = check_tensor(w, 4)) || (rc = check_tensor(y, 4, true))) return rc;
    if (x->dim[1] % groups || w->dim[0] % groups || y->dim[1] != w->dim[0] || x->dim[1] / groups != w->dim[1])
        return PURINE_E_SHAPE;
    if (groups == 1) return PURINE_OK;
    if (!is_float_dtype(x->dtype)) return PURINE_E_DTYPE;
    // every group's slices start on a 16-byte packet (4 floats or 8 bfloat16); the weight and bias
    // gradients are fp32 whatever the activations are
    const int64_t pk = x->dtype == PURINE_BF16 ? 8 : 4;
    const int64_t cg = x->dim[1] / groups, kg = w->dim[0] / groups;
    if ((cg * x->dim[2] * x->dim[3]) % pk || (kg * y->dim[2] * y->dim[3]) % pk ||
        (kg * w->dim[1] * w->dim[2] * w->dim[3]) % pk || kg % pk || nstride_of(x) % pk || nstride_of(y) % pk)
        return PURINE_E_LAYOUT;
    return PURINE_OK;
}

// 2-axis matrices of the fully-connected layer seen by the convolution operators: [rows, features]
// as one image of `rows` channels whose pixel plane is the feature axis, or as a 1x1 filter bank.
purine_tensor as_plane(const purine_tensor* t) {
    purine_tensor v = *t;
    v.ndim = 4; v.dim[0] = 1; v.dim[1] = t->dim[0]; v.dim[2] = 1; v.dim[3] = t->dim[1]; v.nstride = 0;
    return v;
}
purine_tensor as_filter(const purine_tensor* t) {
    purine_tensor v = *t;
    v.ndim = 4; v.dim[0] = t->dim[0]; v.dim[1] = t->dim[1]; v.dim[2] = 1; v.dim[3] = 1; v.nstride = 0;
    return v;
}
const purine_conv_desc kUnitConv{1, 1, 0, 0};

// x, w, y (or dx, w, dy / x, dw, dy for the gradients): 2-axis, of one float dtype; `grad`
// names the fp32 operand of the weight-gradient pass
int check_fc(const purine_tensor* x, const purine_tensor* w, const purine_tensor* y, bool w_is_grad = false) {
    int rc;
    if ((rc = check_tensor(x, 2)) || (rc = check_tensor(w, 2)) || (rc = check_tensor(y, 2))) return rc;
    if (!is_float_dtype(x->dtype) || y->dtype != x->dtype) return PURINE_E_DTYPE;
    if (w->dtype != (w_is_grad ? (int)PURINE_F32 : x->dtype)) return PURINE_E_DTYPE;
    if (x->dim[1] != w->dim[1] || y->dim[0] != x->dim[0] || y->dim[1] != w->dim[0]) return PURINE_E_SHAPE;
    // the reinterpreted descriptors index rows and features with int
    if (x->dim[0] > 0x7fffffff || x->dim[1] > 0x7fffffff || w->dim[0] > 0x7fffffff) return PURINE_E_SHAPE;
    return PURINE_OK;
}
size_t align256(size_t n) { return (n + 255) & ~(size_t)255; }

}  // namespace

size_t purine_grouped_conv_workspace_bytes(int pass, const purine_conv_desc* desc, int groups,
                                           const int64_t x_dim[4], const int64_t w_dim[4], int32_t dtype) {
    if (!x_dim || !w_dim || groups < 1 || x_dim[1] % groups || w_dim[0] % groups) return 0;
    const int64_t xg[4] = {x_dim[0], x_dim[1] / groups, x_dim[2], x_dim[3]};
    const int64_t wg[4] = {w_dim[0] / groups, w_dim[1], w_dim[2], w_dim[3]};
    return purine_conv_workspace_bytes(pass, desc, xg, wg, dtype);
}

int purine_grouped_conv_fwd(const purine_conv_desc* desc, int groups, const purine_tensor* x,
                            const purine_tensor* w, const purine_tensor* b, purine_tensor* y, int relu,
                            void* ws, size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_groups(groups, x, w, y))) return rc;
    if (b && ((rc = check_tensor(b, 1)) || (b->dim[0] != w->dim[0] ? (rc = PURINE_E_SHAPE) : 0))) return rc;
    const int64_t cg = x->dim[1] / groups, kg = w->dim[0] / groups;
    for (int g = 0; g < groups; ++g) {
        const purine_tensor xs = channel_slice(x, g * cg, cg), wsl = row_slice(w, g * kg, kg);
        purine_tensor ys = channel_slice(y, g * kg, kg);
        purine_tensor bs;
        if (b) bs = row_slice(b, g * kg, kg);
        if ((rc = conv_fwd_impl(desc, &xs, &wsl, b ? &bs : nullptr, &ys, relu, ws, ws_bytes, hip_stream))) return rc;
    }
    return PURINE_OK;
}

int purine_grouped_conv_bwd_data(const purine_conv_desc* desc, int groups, const purine_tensor* dy,
                                 const purine_tensor* w, purine_tensor* dx, float beta, void* ws,
                                 size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_groups(groups, dx, w, dy))) return rc;
    const int64_t cg = dx->dim[1] / groups, kg = w->dim[0] / groups;
    for (int g = 0; g < groups; ++g) {
        const purine_tensor dys = channel_slice(dy, g * kg, kg), wsl = row_slice(w, g * kg, kg);
        purine_tensor dxs = channel_slice(dx, g * cg, cg);
        if ((rc = conv_bwd_data_impl(desc, &dys, &wsl, nullptr, &dxs, beta, ws, ws_bytes, hip_stream))) return rc;
    }
    return PURINE_OK;
}

int purine_grouped_conv_bwd_weight(const purine_conv_desc* desc, int groups, const purine_tensor* x,
                                   const purine_tensor* dy, purine_tensor* dw, purine_tensor* db,
                                   float beta, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_groups(groups, x, dw, dy))) return rc;
    if (db && ((rc = check_tensor(db, 1)) || (db->dim[0] != dw->dim[0] ? (rc = PURINE_E_SHAPE) : 0))) return rc;
    const int64_t cg = x->dim[1] / groups, kg = dw->dim[0] / groups;
    for (int g = 0; g < groups; ++g) {
        const purine_tensor xs = channel_slice(x, g * cg, cg), dys = channel_slice(dy, g * kg, kg);
        purine_tensor dws = row_slice(dw, g * kg, kg);
        purine_tensor dbs;
        if (db) dbs = row_slice(db, g * kg, kg);
        if ((rc = conv_bwd_weight_impl(desc, &xs, &dys, &dws, db ? &dbs : nullptr, beta, ws, ws_bytes, hip_stream)))
            return rc;
    }
    return PURINE_OK;
}

size_t purine_fc_workspace_bytes(int pass, int64_t N, int64_t C, int64_t K, int32_t dtype) {
    if (N < 1 || C < 1 || K < 1 || !is_float_dtype(dtype)) return 0;
    // one convolution geometry serves the three fp32 passes: a 1x1 filter bank [N, K] over the plane [1, K, 1, C]
    const int64_t xd[4] = {1, K, 1, C}, wd[4] = {N, K, 1, 1};
    switch (pass) {
        case PURINE_CONV_FWD:   // y = x w^T through the weight-gradient kernel (split reduction over C)
            return align256(purine_conv_workspace_bytes(PURINE_CONV_BWD_WEIGHT, &kUnitConv, xd, wd, dtype)) +
                   (dtype == PURINE_BF16 ? (size_t)N * K * 4 : 0);   // bf16: the fp32 product matrix before the bias
        case PURINE_CONV_BWD_DATA: {   // dx = dy w through the forward kernel, or (bf16) a kernel of its own
            const size_t own = dtype == PURINE_BF16 ? fc_dgrad_bf16_plan(N, C, K, nullptr, nullptr) : SIZE_MAX;
            return own != SIZE_MAX ? own : purine_conv_workspace_bytes(PURINE_CONV_FWD, &kUnitConv, xd, wd, dtype);
        }
        case PURINE_CONV_BWD_WEIGHT:
        case PURINE_CONV_BWD_WEIGHT_BIAS: {
            if (dtype == PURINE_BF16) {
                // dw = dy^T x through the weight-gradient kernel on the transposed matrices (the batch
                // as the pixel axis): both transposes and that kernel's partial sums
                const int64_t xt[4] = {1, C, 1, N}, wt[4] = {K, C, 1, 1};
                return align256((size_t)N * C * 2) + align256((size_t)N * K * 2) +
                       align256(purine_conv_workspace_bytes(PURINE_CONV_BWD_WEIGHT, &kUnitConv, xt, wt, dtype));
            }
            // fp32: dw = dy^T x through the backward-data kernel; db needs no scratch
            return align256(purine_conv_workspace_bytes(PURINE_CONV_BWD_DATA, &kUnitConv, xd, wd, dtype));
        }
        default: return 0;
    }
}

int purine_fc_fwd(const purine_tensor* x, const purine_tensor* w, const purine_tensor* b, purine_tensor* y,
                  void* ws, size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_fc(x, w, y))) return rc;
    if (b) {
        if ((rc = check_tensor(b, 1))) return rc;
        if (b->dtype != y->dtype) return PURINE_E_DTYPE;
        if (b->dim[0] != w->dim[0]) return PURINE_E_SHAPE;
        if (overlaps(b, y)) return PURINE_E_LAYOUT;
    }
    // y[n][k] = sum_c x[n][c] w[k][c]: the weight-gradient contraction with dy := x and x := w,
    // both matrices as one image whose pixel plane is the feature axis c
    const purine_tensor wp = as_plane(w), xp = as_plane(x);
    purine_tensor yf = as_filter(y);
    if (x->dtype == PURINE_BF16) {
        // that kernel's result is fp32: it goes to the end of the workspace, and a last kernel adds
        // the bias and rounds once
        const int64_t N = x->dim[0], K = w->dim[0];
        const size_t conv_ws = align256(purine_conv_workspace_bytes(PURINE_CONV_BWD_WEIGHT, &kUnitConv, wp.dim, yf.dim, PURINE_BF16));
        if (!ws || ws_bytes < conv_ws + (size_t)N * K * 4) return PURINE_E_WORKSPACE;
        if (((uintptr_t)ws) & 15u) return PURINE_E_LAYOUT;
        purine_tensor acc = yf;
        acc.dtype = PURINE_F32;
        acc.data = (char*)ws + conv_ws;
        if ((rc = conv_bwd_weight_impl(&kUnitConv, &wp, &xp, &acc, nullptr, 0.0f, ws, conv_ws, hip_stream))) return rc;
        return hip_status(launch_fc_finish_bf16((const float*)acc.data, b ? b->data : nullptr, y->data, (int)N, (int)K,
                                                (hipStream_t)hip_stream));
    }
    if ((rc = conv_bwd_weight_impl(&kUnitConv, &wp, &xp, &yf, nullptr, 0.0f, ws, ws_bytes, hip_stream))) return rc;
    if (b)
        return hip_status(launch_bias_rows((const float*)b->data, (float*)y->data, (int)y->dim[0], (int)y->dim[1],
                                           (hipStream_t)hip_stream));
    return PURINE_OK;
}

int purine_fc_bwd_data(const purine_tensor* dy, const purine_tensor* w, purine_tensor* dx, void* ws,
                       size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_fc(dx, w, dy))) return rc;
    // dx[n][c] = sum_k dy[n][k] w[k][c]: a 1x1 convolution of the plane w [K channels x C pixels] with
    // the filter bank dy [N x K]
    if (dy->dtype == PURINE_BF16) {
        // rows of whole 16-byte packets: the kernel that stages w as it lies in memory
        const size_t need = fc_dgrad_bf16_plan(dy->dim[0], w->dim[1], w->dim[0], nullptr, nullptr);
        if (need != SIZE_MAX) {
            if (overlaps(dx, dy) || overlaps(dx, w)) return PURINE_E_LAYOUT;
            if (need && (!ws || ws_bytes < need)) return PURINE_E_WORKSPACE;
            if (need && (((uintptr_t)ws) & 15u)) return PURINE_E_LAYOUT;
            return hip_status(launch_fc_dgrad_bf16(dy->data, w->data, dx->data, (int)dy->dim[0], (int)w->dim[0],
                                                   (int)w->dim[1], ws, (hipStream_t)hip_stream));
        }
    }
    const purine_tensor wp = as_plane(w), dyf = as_filter(dy);
    purine_tensor dxp = as_plane(dx);
    return conv_fwd_impl(&kUnitConv, &wp, &dyf, nullptr, &dxp, 0, ws, ws_bytes, hip_stream);
}

int purine_fc_bwd_weight(const purine_tensor* x, const purine_tensor* dy, purine_tensor* dw, purine_tensor* db,
                         float beta, void* ws, size_t ws_bytes, void* hip_stream) {
    int rc;
    if ((rc = check_fc(x, dw, dy, true)) || (rc = check_beta(beta))) return rc;
    const int64_t N = x->dim[0], C = x->dim[1], K = dw->dim[0];
    const purine_tensor dy4 = as_filter(dy);
    if (db) {
        if ((rc = check_tensor(db, 1))) return rc;
        if (db->dtype != PURINE_F32) return PURINE_E_DTYPE;
        if (db->dim[0] != dw->dim[0]) return PURINE_E_SHAPE;
        if (overlaps(db, dy) || overlaps(db, x) || overlaps(db, dw)) return PURINE_E_LAYOUT;
    }
    if (x->dtype == PURINE_BF16) {
        // dw[k][c] = sum_n dy[n][k] x[n][c] with an fp32 result: the weight-gradient contraction over
        // the batch as the pixel axis, on transposed copies x^T [C x N] and dy^T [K x N]
        const int64_t xt[4] = {1, C, 1, N}, wt[4] = {K, C, 1, 1};
        const size_t xt_bytes = align256((size_t)N * C * 2), dyt_bytes = align256((size_t)N * K * 2);
        const size_t wg_ws = align256(purine_conv_workspace_bytes(PURINE_CONV_BWD_WEIGHT, &kUnitConv, xt, wt, PURINE_BF16));
        if (!ws || ws_bytes < xt_bytes + dyt_bytes + wg_ws) return PURINE_E_WORKSPACE;
        if (((uintptr_t)ws) & 15u) return PURINE_E_LAYOUT;
        if (overlaps(dw, x) || overlaps(dw, dy)) return PURINE_E_LAYOUT;
        purine_tensor xT = *x, dyT = *dy;
        xT.data = ws; dyT.data = (char*)ws + xt_bytes;
        xT.dim[0] = C; xT.dim[1] = N; dyT.dim[0] = K; dyT.dim[1] = N;
        hipError_t e = launch_transpose16_pair(x->data, xT.data, (int)C, dy->data, dyT.data, (int)K, (int)N,
                                               (hipStream_t)hip_stream);
        if (e != hipSuccess) return hip_status(e);
        if (fc_wgrad_bf16_applies(N, C, K)) {
            // batches of whole 16-byte packets: one kernel that owns whole tiles of dw (no partial sums)
            e = launch_fc_wgrad_bf16(dyT.data, xT.data, (float*)dw->data, (int)N, (int)K, (int)C, beta != 0.0f,
                                     (hipStream_t)hip_stream);
            if (e != hipSuccess) return hip_status(e);
        } else {
            const purine_tensor xp = as_plane(&xT), dyp = as_plane(&dyT);
            purine_tensor dwf = as_filter(dw);
            if ((rc = conv_bwd_weight_impl(&kUnitConv, &xp, &dyp, &dwf, nullptr, beta, (char*)ws + xt_bytes + dyt_bytes,
                                           wg_ws, hip_stream)))
                return rc;
        }
    } else {
        // dw[k][c] = sum_n dy[n][k] x[n][c]: the backward-data contraction with dy := x (plane of N
        // channels) and w := dy (filter bank [N x K])
        const purine_tensor xp = as_plane(x);
        purine_tensor dwp = as_plane(dw);
        if ((rc = conv_bwd_data_impl(&kUnitConv, &xp, &dy4, nullptr, &dwp, beta, ws, ws_bytes, hip_stream))) return rc;
    }
    if (db)   // column sums of dy
        return hip_status(launch_fc_bias_bwd(dy->dtype, dy->data, (float*)db->data, (int)N, (int)K, beta,
                                             (hipStream_t)hip_stream));
    return PURINE_OK;
}

// Tuning hook: force the tile shape of the forward / backward-data kernels (0, 0 = automatic).
void purine_debug_force_tile(int bm, int bn) { force_pix_tile(bm, bn); }

// Test hook for the host-side reciprocal division used by the kernels' index arithmetic.
uint32_t purine_debug_fastdiv(uint32_t n, uint32_t d) { return fastdiv(n, make_fastdiv(d)); }

}  // extern "C"

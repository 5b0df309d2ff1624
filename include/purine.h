/*
 * purine.h - C ABI of the MI355X (gfx950) convolution-layer operator library and of the minimal
 * single-GPU bi-graph executor.
 *
 * The library implements the operators inside the convolution layer of the paper's Figure 1(b)
 * (section 2: a network is a bipartite graph of tensors and operators; "operators are functions
 * of the incoming tensors and the results are put in the outgoing tensors"), and the event-driven
 * task dispatcher of section 2.1 restricted to one GPU, with the `thread` property of section 3
 * mapped to HIP streams.
 *
 * Conventions that hold for every entry point unless stated otherwise
 *   - All tensor data pointers are DEVICE pointers (HBM), owned by the caller. The library never
 *     allocates or frees device memory; scratch comes in through `ws`, whose size the matching
 *     *_workspace_bytes query returns. Descriptor structs and dimension arrays are HOST memory,
 *     read during the call only.
 *   - Tensors are dense, row-major: activations NCHW, filters KCRS, bias [K]. `dim` holds the
 *     extents, outermost first; unused trailing entries are ignored. No tensor may hold 2^31 or
 *     more elements. Data pointers must be aligned to 16 bytes. One tighter limit: a PURINE_BF16
 *     convolution or backward-data pass whose filter has more than one tap and at least 16
 *     channels on the gathered side, and whose gathered tensor (x, or dy for backward-data) has
 *     rows that are not whole 16-byte packets (W not a multiple of 8, or a channel count or image
 *     stride not a multiple of 8), stages a channels-blocked copy of that tensor (channels rounded
 *     up to a multiple of 32) in ws, and that copy must stay below 2^31 bytes, i.e. 2^30 elements
 *     (PURINE_E_SHAPE otherwise). Layers with whole-packet rows are read in place.
 *   - Channel-slice views: a 4-axis F32 or BF16 activation tensor may set `nstride`, the distance in
 *     elements between consecutive images, to more than C*H*W: the tensor is then channels
 *     c0..c0+C-1 of a larger NCHW buffer with `data` pointing at channel c0 of image 0 (inside an
 *     image the layout stays dense). nstride must be a whole number of 16-byte packets (a
 *     multiple of 4 for F32, of 8 for BF16) and the span
 *     (N-1)*nstride + C*H*W must stay below 2^31 elements. Views are accepted where an entry
 *     point says so (the activation arguments of the convolution operators and of ReLU); every
 *     other argument must be dense (PURINE_E_LAYOUT otherwise). Two views of one buffer with the
 *     same nstride overlap only if their channel ranges do.
 *   - dtype: PURINE_F32 tensors hold IEEE binary32. PURINE_BF16 tensors hold bfloat16 bit
 *     patterns (uint16); arithmetic accumulates in fp32; results stored as bf16 are rounded to
 *     nearest even. Weight and bias gradients are always PURINE_F32.
 *   - Operator calls validate their arguments first (no launch happens on error), enqueue their
 *     kernels on `hip_stream` (a hipStream_t passed as void*; NULL = the null stream) and return
 *     without waiting. Only purine_graph_run blocks.
 *   - Return value: PURINE_OK (0) or a negative purine_status. Nothing aborts or throws.
 *   - beta is 0 (overwrite the output) or 1 (add to what the output already holds).
 *   - Results are deterministic: the same inputs give bit-identical outputs run to run (no
 *     floating-point atomics; split reductions are summed in a fixed order).
 */
#ifndef PURINE_H
#define PURINE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum { PURINE_F32 = 0, PURINE_BF16 = 1, PURINE_I32 = 2 } purine_dtype;

typedef enum {
    PURINE_OK = 0,
    PURINE_E_NULL = -1,      /* a required pointer is NULL                                  */
    PURINE_E_SHAPE = -2,     /* extents inconsistent, empty, or too large                   */
    PURINE_E_DTYPE = -3,     /* unsupported dtype or dtype combination                      */
    PURINE_E_LAYOUT = -4,    /* misaligned data pointer or illegal aliasing                 */
    PURINE_E_WORKSPACE = -5, /* ws is NULL or smaller than the query says                   */
    PURINE_E_GRAPH = -6,     /* not a legal bi-graph (see purine_graph_run)                 */
    PURINE_E_HIP = -7,       /* the HIP runtime reported an error                           */
    PURINE_E_ARG = -8,       /* a scalar argument is out of range (stride, beta, ids, ...)  */
    PURINE_E_STATIC_SCRATCH = -9 /* purine_conv_bwd_weight_static: the layer needs more scratch
                                    than purine_static_scratch_bytes()                         */
} purine_status;

typedef struct {
    void*   data;   /* device pointer                                  */
    int32_t dtype;  /* purine_dtype                                    */
    int32_t ndim;   /* 1..4                                            */
    int64_t dim[4]; /* extents, outermost first                        */
    int64_t nstride; /* 0 (dense) or elements between images, see above */
} purine_tensor;

/* Convolution geometry. Filter extents R,S and the channel counts come from the filter tensor.
 * Cross-correlation (no kernel flip), symmetric zero padding, no dilation, one group.
 * Output extent along an axis: floor((in + 2*pad - k)/stride) + 1. */
typedef struct { int32_t stride_h, stride_w, pad_h, pad_w; } purine_conv_desc;

/* Square max-pooling window. */
typedef struct { int32_t window, stride, pad; } purine_pool_desc;

typedef enum {
    PURINE_CONV_FWD = 0, PURINE_CONV_BWD_DATA = 1, PURINE_CONV_BWD_WEIGHT = 2,
    PURINE_CONV_BWD_WEIGHT_BIAS = 3   /* purine_conv_bwd_weight_bias: both sets of partial sums */
} purine_conv_pass;

const char* purine_status_string(int status);
/* Name of the HIP error behind the last PURINE_E_HIP returned to this host thread. */
const char* purine_last_hip_error(void);

/* y_dim = {N, K, P, Q} for x_dim = {N, C, H, W}, w_dim = {K, C, R, S}.
 * PURINE_E_SHAPE when channels disagree, an extent is < 1, or the padded input is smaller than the
 * filter; PURINE_E_ARG when a stride is < 1 or a pad is < 0. Pure host integer code. */
int purine_conv_out_shape(const purine_conv_desc* desc, const int64_t x_dim[4],
                          const int64_t w_dim[4], int64_t y_dim[4]);

/* Bytes of device scratch the given pass needs (0 when none). Returns 0 for illegal shapes: the
 * operator call itself reports the error. Forward and backward-data keep a repacked, zero-padded
 * copy of the filter there (none for a forward pass with fewer than 16 input channels);
 * backward-weight keeps its split-reduction partial sums there. */
size_t purine_conv_workspace_bytes(int pass, const purine_conv_desc* desc, const int64_t x_dim[4],
                                   const int64_t w_dim[4], int32_t dtype);
size_t purine_bias_bwd_workspace_bytes(const int64_t dy_dim[4], int32_t dtype);

/* ---- the five operators of the convolution layer (paper Figure 1(b)) ---------------------- */

/* Conv: y[n,k,p,q] = sum_{c,r,s} x[n,c,p*sh-ph+r,q*sw-pw+s] * w[k,c,r,s], taps outside x are 0.
 * x, w, y share one dtype (F32 or BF16). The patch matrix is never written to memory.
 * ws: scratch of at least purine_conv_workspace_bytes(PURINE_CONV_FWD, ...) bytes (may be NULL when
 * that is 0); it must not overlap any tensor. y must not overlap x or w. */
int purine_conv_fwd(const purine_conv_desc* desc, const purine_tensor* x, const purine_tensor* w,
                    purine_tensor* y, void* ws, size_t ws_bytes, void* hip_stream);

/* ConvBwdData: dx[n,c,h,w] = beta*dx + sum over (k,r,s,p,q) with p*sh-ph+r = h, q*sw-pw+s = w of
 * dy[n,k,p,q] * w[k,c,r,s]. dy, w, dx share one dtype. dx's extents must be the x extents whose
 * forward output has dy's extents. ws as for the forward pass (query with PURINE_CONV_BWD_DATA). */
int purine_conv_bwd_data(const purine_conv_desc* desc, const purine_tensor* dy,
                         const purine_tensor* w, purine_tensor* dx, float beta, void* ws,
                         size_t ws_bytes, void* hip_stream);

/* Fused operator vertices (an operator is any function of its incoming tensors, section 2): the
 * same kernels with the elementwise neighbours of Figure 1(b) folded into their epilogues, which
 * saves one read and one write of the whole activation tensor per folded operator.
 *   purine_conv_fwd_bias_relu : y = conv(x, w) + b[k]  (b may be NULL), then y = max(y, 0) if relu = 1.
 *   purine_conv_bwd_data_relu : dx = beta*dx + (act > 0 ? ConvBwdData(dy, w) : 0); act has dx's
 *       extents and dtype and is the OUTPUT of the ReLU that produced this layer's input (the ReLU
 *       gradient of the layer below, applied where its input gradient is produced). */
int purine_conv_fwd_bias_relu(const purine_conv_desc* desc, const purine_tensor* x,
                              const purine_tensor* w, const purine_tensor* b, purine_tensor* y,
                              int relu, void* ws, size_t ws_bytes, void* hip_stream);
int purine_conv_bwd_data_relu(const purine_conv_desc* desc, const purine_tensor* dy,
                              const purine_tensor* w, const purine_tensor* act, purine_tensor* dx,
                              float beta, void* ws, size_t ws_bytes, void* hip_stream);

/* ConvBwdWeight: dw[k,c,r,s] = beta*dw + sum_{n,p,q} dy[n,k,p,q] * x[n,c,p*sh-ph+r,q*sw-pw+s].
 * A plain sum over the batch (no 1/N), so shards of a data-parallel minibatch add up
 * (paper section 3.4). x and dy share one dtype; dw is F32. The pixel reduction is split into
 * chunks whose fp32 partial sums go to ws and are added in chunk order by a second kernel. */
int purine_conv_bwd_weight(const purine_conv_desc* desc, const purine_tensor* x,
                           const purine_tensor* dy, purine_tensor* dw, float beta, void* ws,
                           size_t ws_bytes, void* hip_stream);

/* ConvBwdWeight for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. Same operator, same
 * kernels and bit-identical results as purine_conv_bwd_weight, but the split-reduction partial
 * sums go to a fixed array inside the library's device image (purine_static_scratch_bytes() bytes,
 * 64 MiB, held by every GPU the library runs on until the process ends). The call allocates
 * nothing: no hipMalloc / hipFree and no allocating library routine. A layer whose
 * purine_conv_workspace_bytes(PURINE_CONV_BWD_WEIGHT, ...) exceeds that size is refused with
 * PURINE_E_STATIC_SCRATCH before anything is launched. The first call on a device looks up that
 * device's address of the array (once; the device current at the call is the one used). Every
 * call on a GPU shares that GPU's array: calls that overlap in time on one GPU (different streams
 * with no ordering between them, or different host threads) race on it and must be ordered by the
 * caller; nothing needs clearing between calls (each call writes every partial sum it later reads). */
int purine_conv_bwd_weight_static(const purine_conv_desc* desc, const purine_tensor* x,
                                  const purine_tensor* dy, purine_tensor* dw, float beta,
                                  void* hip_stream);
size_t purine_static_scratch_bytes(void);

/* ConvBwdWeight and BiasBwd of one layer as a single operator (both read all of dy; paper
 * Figure 1(b) draws them as two vertices on the same incoming tensor): dw as above and
 * db[k] = beta*db + sum_{n,p,q} dy[n,k,p,q], db F32 of K elements. The dy fragments that feed the
 * matrix cores are summed on the way, so dy is read once. Partial sums per chunk for both, added
 * in chunk order by the second kernel. ws: purine_conv_workspace_bytes(PURINE_CONV_BWD_WEIGHT_BIAS).
 * db must not overlap x, dy or dw. */
int purine_conv_bwd_weight_bias(const purine_conv_desc* desc, const purine_tensor* x,
                                const purine_tensor* dy, purine_tensor* dw, purine_tensor* db,
                                float beta, void* ws, size_t ws_bytes, void* hip_stream);

/* Bias: y[n,k,p,q] += b[k], in place. y: F32 or BF16 (add in fp32); b: same dtype as y. */
int purine_bias_fwd(const purine_tensor* b, purine_tensor* y, void* hip_stream);

/* BiasBwd: db[k] = beta*db + sum_{n,p,q} dy[n,k,p,q]. db is F32. Two-level fixed-order sum. */
int purine_bias_bwd(const purine_tensor* dy, purine_tensor* db, float beta, void* ws,
                    size_t ws_bytes, void* hip_stream);

/* ---- exact support operators that chain conv layers into the synthetic workloads ---------- */

/* y = max(x, 0). y may be x itself. Same dtype and extents. */
int purine_relu_fwd(const purine_tensor* x, purine_tensor* y, void* hip_stream);
/* dx = dy where x > 0, else 0. x may be the forward input or output (same sign test).
 * dx may be dy itself. */
int purine_relu_bwd(const purine_tensor* x, const purine_tensor* dy, purine_tensor* dx,
                    void* hip_stream);
/* Max pooling. Padded positions never win; ties go to the first maximum in row-major window
 * order. arg (I32, extents of y) receives the winner's flat position h*W+w inside its plane. */
int purine_maxpool_fwd(const purine_pool_desc* desc, const purine_tensor* x, purine_tensor* y,
                       purine_tensor* arg, void* hip_stream);
/* dx[n,c,arg] = beta*dx + sum of dy over the windows that chose that position (fp32 sum, windows
 * taken in row-major order). */
int purine_maxpool_bwd(const purine_pool_desc* desc, const purine_tensor* dy,
                       const purine_tensor* arg, purine_tensor* dx, float beta, void* hip_stream);
/* The same followed by the ReLU gradient of the pooled tensor, as one operator (fusion in the
 * sense of paper section 3.4's note that adjacent operators may share a kernel). y: the pooling
 * output of the forward pass (extents and dtype of dy). Only windows with y > 0 pass their dy on:
 * dx[n,c,pos] = beta*dx + sum of dy over the windows that chose pos and have y > 0, same order of
 * summation. A position that won a window holds that window's y, so when the pooled tensor is a
 * ReLU output this is purine_maxpool_bwd followed by purine_relu_bwd on it: bit for bit the former
 * where the pooled tensor is positive, beta*dx elsewhere. The pooled tensor itself is not read. */
int purine_maxpool_bwd_relu(const purine_pool_desc* desc, const purine_tensor* dy,
                            const purine_tensor* arg, const purine_tensor* y, purine_tensor* dx,
                            float beta, void* hip_stream);
/* Channel concatenation of n_parts NCHW tensors (same N,H,W,dtype) and its inverse. */
int purine_concat_fwd(const purine_tensor* const* parts, int n_parts, purine_tensor* out,
                      void* hip_stream);
int purine_concat_bwd(const purine_tensor* dout, purine_tensor* const* dparts, int n_parts,
                      void* hip_stream);
/* out = terms[0] + terms[1] + ... in that order, fp32 adds (gradient fan-in). 1 <= n_terms <= 8.
 * out may be terms[0]. */
int purine_sum(const purine_tensor* const* terms, int n_terms, purine_tensor* out,
               void* hip_stream);

/* SGD step on one parameter tensor (paper section 2.2, Figure 2(a): the network graph leaves the
 * updated parameters in a separate "new params" tensor so that the graph stays acyclic):
 * new_w = w - lr * dw, element by element, one fused multiply-add in fp32 (bf16 parameters are
 * widened, updated, and rounded to nearest even). w and new_w: same dtype (F32 or BF16) and
 * extents, 1 to 4 axes; dw: F32, same extents. new_w may be w itself (update in place) but may
 * not overlap it partially, nor dw. */
int purine_sgd_update(const purine_tensor* w, const purine_tensor* dw, purine_tensor* new_w,
                      float lr, void* hip_stream);

/* ---- grouped convolution and fully-connected layer (the other layer types of the networks the
 *      paper's parallelisation schemes are discussed on, section 3): compositions of the operators
 *      above, no kernels of their own ---------------------------------------------------------- */

/* Grouped convolution: x [N,C,H,W], w [K, C/G, R, S], y [N,K,P,Q]; output channels
 * g*K/G .. (g+1)*K/G-1 see only input channels g*C/G .. (g+1)*C/G-1. Runs the matching operator once
 * per group on channel-slice views of x, y (dy, dx) and on the group's rows of w (b, dw, db), one
 * group after the other on the stream, all sharing ws (purine_grouped_conv_workspace_bytes: one
 * group's need). groups = 1 is the plain operator. For groups > 1: (C/G)*H*W, (K/G)*P*Q,
 * (K/G)*(C/G)*R*S and K/G must be multiples of 4 (F32 activations) or 8 (BF16) so that every
 * slice keeps the alignment rules (PURINE_E_LAYOUT otherwise). b and db may be NULL. x, y, dy, dx may themselves
 * be views. */
size_t purine_grouped_conv_workspace_bytes(int pass, const purine_conv_desc* desc, int groups,
                                           const int64_t x_dim[4], const int64_t w_dim[4],
                                           int32_t dtype);
int purine_grouped_conv_fwd(const purine_conv_desc* desc, int groups, const purine_tensor* x,
                            const purine_tensor* w, const purine_tensor* b, purine_tensor* y,
                            int relu, void* ws, size_t ws_bytes, void* hip_stream);
int purine_grouped_conv_bwd_data(const purine_conv_desc* desc, int groups, const purine_tensor* dy,
                                 const purine_tensor* w, purine_tensor* dx, float beta, void* ws,
                                 size_t ws_bytes, void* hip_stream);
int purine_grouped_conv_bwd_weight(const purine_conv_desc* desc, int groups, const purine_tensor* x,
                                   const purine_tensor* dy, purine_tensor* dw, purine_tensor* db,
                                   float beta, void* ws, size_t ws_bytes, void* hip_stream);

/* Fully-connected layer on dense 2-axis matrices: x [N,C], w [K,C], b [K], y [N,K], all F32 or all
 * BF16; dw and db are F32.
 *   fwd:        y = x w^T (+ b)          dx = dy w          dw = beta*dw + dy^T x,  db = beta*db + column sums of dy
 * Each pass is one of the convolution GEMM kernels on reinterpreted descriptors (a matrix
 * [rows, features] is one image of `rows` channels whose pixel plane is the feature axis, or a 1x1
 * filter bank): forward runs the weight-gradient kernel (split reduction over C, fixed-order
 * second pass; BF16: its fp32 result gets the bias added and is rounded once), backward-data the
 * forward kernel (with a split reduction over K when its tiles alone would leave most of the chip
 * idle), backward-weight the backward-data kernel (F32) or, for BF16 (the result is fp32), a
 * contraction over the batch on transposed copies of x and dy kept in ws: a kernel that owns whole
 * tiles of dw when N is a multiple of 8, else the weight-gradient kernel with the batch as the
 * pixel axis. db is a column-sum kernel of its own (fixed summation order).
 * pass for the workspace query: PURINE_CONV_FWD, _BWD_DATA, _BWD_WEIGHT. b and db may be NULL. */
size_t purine_fc_workspace_bytes(int pass, int64_t N, int64_t C, int64_t K, int32_t dtype);
int purine_fc_fwd(const purine_tensor* x, const purine_tensor* w, const purine_tensor* b,
                  purine_tensor* y, void* ws, size_t ws_bytes, void* hip_stream);
int purine_fc_bwd_data(const purine_tensor* dy, const purine_tensor* w, purine_tensor* dx, void* ws,
                       size_t ws_bytes, void* hip_stream);
int purine_fc_bwd_weight(const purine_tensor* x, const purine_tensor* dy, purine_tensor* dw,
                         purine_tensor* db, float beta, void* ws, size_t ws_bytes, void* hip_stream);

/* ---- bi-graph executor (paper sections 2, 2.1, 2.2 and the `thread` property of section 3) -- */

typedef struct purine_graph purine_graph;

typedef enum {
    PURINE_OP_CONV_FWD = 0,        /* in: x, w            out: y                                 */
    PURINE_OP_BIAS_FWD = 1,        /* in: y, b            out: y' (same storage as y)            */
    PURINE_OP_CONV_BWD_DATA = 2,   /* in: dy, w [, dx]    out: dx'   (third input iff beta = 1)  */
    PURINE_OP_CONV_BWD_WEIGHT = 3, /* in: x, dy [, dw]    out: dw'                               */
    PURINE_OP_BIAS_BWD = 4,        /* in: dy [, db]       out: db'                               */
    PURINE_OP_RELU_FWD = 5,        /* in: x               out: y                                 */
    PURINE_OP_RELU_BWD = 6,        /* in: x, dy           out: dx                                */
    PURINE_OP_MAXPOOL_FWD = 7,     /* in: x               out: y, arg                            */
    PURINE_OP_MAXPOOL_BWD = 8,     /* in: dy, arg [, dx]  out: dx'                               */
    PURINE_OP_CONCAT_FWD = 9,      /* in: parts...        out: cat                               */
    PURINE_OP_CONCAT_BWD = 10,     /* in: dcat            out: dparts...                         */
    PURINE_OP_SUM = 11,            /* in: terms...        out: sum                               */
    PURINE_OP_HOST_NOP = 12,       /* any in/out; does nothing on the device (bookkeeping tests) */
    PURINE_OP_CONV_FWD_BIAS_RELU = 13, /* in: x, w, b     out: y   (attrs.relu selects the ReLU)    */
    PURINE_OP_CONV_BWD_DATA_RELU = 14, /* in: dy, w, act [, dx]  out: dx'                           */
    PURINE_OP_CONV_BWD_WEIGHT_BIAS = 15, /* in: x, dy [, dw, db]  out: dw', db'                      */
    PURINE_OP_SGD_UPDATE = 16,         /* in: w, dw           out: new_w   (attrs.lr)                */
    PURINE_OP_ALIAS = 17,              /* in: 1..64 tensors   out: 1..64 tensors inside their storage */
    PURINE_OP_FC_FWD = 18,             /* in: x, w, b         out: y                                 */
    PURINE_OP_FC_BWD_DATA = 19,        /* in: dy, w           out: dx                                */
    PURINE_OP_FC_BWD_WEIGHT = 20,      /* in: x, dy [, dw, db]  out: dw', db'                        */
    PURINE_OP_GROUPED_CONV_FWD = 21,   /* in: x, w, b         out: y   (attrs.groups, attrs.relu)    */
    PURINE_OP_GROUPED_CONV_BWD_DATA = 22,   /* in: dy, w [, dx]      out: dx'  (attrs.groups)        */
    PURINE_OP_GROUPED_CONV_BWD_WEIGHT = 23, /* in: x, dy [, dw, db]  out: dw', db'  (attrs.groups)   */
    PURINE_OP_MAXPOOL_BWD_RELU = 24         /* in: dy, arg, y [, dx]    out: dx'                     */
} purine_op_kind;

/* PURINE_OP_ALIAS does no device work. It gives storage that other operators have written a tensor
 * vertex of its own: channel slices of a buffer one operator filled (one input, several outputs),
 * or the buffer that several operators filled slice by slice (several inputs, one output: the
 * concatenation, with no copy). Every output must lie inside the span of the inputs
 * (PURINE_E_LAYOUT from purine_graph_add_op otherwise). It fires like a device operator: its
 * outputs become ready, in stream order, once all its inputs are. */

typedef struct {
    purine_conv_desc conv;   /* conv ops                                          */
    purine_pool_desc pool;   /* pool ops                                          */
    float  beta;             /* ops with an accumulate form                       */
    int32_t relu;            /* PURINE_OP_CONV_FWD_BIAS_RELU: apply max(y, 0)     */
    void*  ws;               /* device scratch private to this operator           */
    size_t ws_bytes;
    float  lr;               /* PURINE_OP_SGD_UPDATE: step size                   */
    int32_t groups;          /* grouped convolution ops (0 is read as 1)          */
} purine_op_attrs;

/* The graph owns only host bookkeeping plus the HIP streams and events it creates lazily (none for
 * a graph of HOST_NOP operators, so such graphs run on a machine without a GPU). */
purine_graph* purine_graph_create(void);
void purine_graph_destroy(purine_graph* g);

/* Adds a tensor vertex; the descriptor is copied. name may be NULL. Returns the tensor id (>= 0)
 * or a negative status. Two vertices may share storage: a tensor vertex is one VERSION of a
 * buffer (an in-place operator reads version i and writes version i+1 at the same address). A
 * vertex may have several incoming operators; it is ready when all of them are done (section 2.1). */
int purine_graph_add_tensor(purine_graph* g, const purine_tensor* t, const char* name);

/* Adds an operator vertex with edges in_ids -> op -> out_ids (edges only ever join a tensor and an
 * operator, section 2). thread_id >= 0: operators with the same id are issued in order on one
 * HIP stream; different ids may overlap (section 3). attrs may be NULL for kinds that need none.
 * Returns the operator id (>= 0) or a negative status (bad ids, wrong arity for the kind). */
int purine_graph_add_op(purine_graph* g, int op_kind, const purine_op_attrs* attrs,
                        const int* in_ids, int n_in, const int* out_ids, int n_out, int thread_id);

/* Binds a thread id to a caller-owned hipStream_t (otherwise the graph creates one on first use). */
int purine_graph_set_stream(purine_graph* g, int thread_id, void* hip_stream);

/* Checks the graph without running it: acyclic; every tensor with no incoming operator is a source
 * (ready at start); any two operators that touch overlapping storage, at least one of them
 * writing, are ordered by a path in the graph. PURINE_E_GRAPH otherwise. */
int purine_graph_validate(purine_graph* g);

/* Runs the graph once (section 2.1): starts from the source tensors, fires an operator when all its
 * incoming tensors are ready, marks a tensor ready when all its incoming operators have been
 * issued (stream order plus events carry the readiness onto the device), and returns when every
 * sink has been reached and the device work behind it has completed - the synchronisation point
 * that lets graphs be iterated (section 2.2). Work the caller enqueued earlier on other streams
 * must have completed before the call. A graph that cannot reach its sinks returns
 * PURINE_E_GRAPH instead of hanging. The first operator error aborts the run and is returned. */
int purine_graph_run(purine_graph* g);

/* The swap step of graph iteration (section 2.2, Figure 2(b)): exchanges the storage addresses of
 * two tensor vertices with the same dtype and extents ("old" and "new" parameters), so that the
 * next run of the graph reads what the last run wrote. Every vertex bound to either address moves
 * with it. PURINE_E_SHAPE when the two differ in dtype or extents; PURINE_E_LAYOUT when the two
 * ranges overlap, or some other vertex or operator scratch overlaps one of them without covering
 * exactly the same bytes (the exchange would then change which operators conflict). Host only;
 * call between runs. */
int purine_graph_swap_storage(purine_graph* g, int tensor_a, int tensor_b);
/* Storage address a tensor vertex is bound to at the moment (NULL for a bad id). */
void* purine_graph_tensor_data(const purine_graph* g, int tensor_id);

/* Graph iteration (section 2.2, Figure 2(c)): n_iters times { one run of the graph; then
 * purine_graph_swap_storage(swap_a[i], swap_b[i]) for i < n_swaps }. The end of each run is the
 * synchronisation point between iterations, and the device keeps it: no operator of an iteration
 * starts before every operator of the one before has finished (each stream waits for all the
 * others), while the host goes on issuing and waits once, after the last iteration; results are
 * those of n_iters calls of purine_graph_run with the swaps between them. Host operators wait for
 * their device producers as in a single run. The firing log and the timing brackets are those of
 * the last iteration. Stops issuing at the first error, waits for what was issued and returns
 * the error. */
int purine_graph_iterate(purine_graph* g, int n_iters, const int* swap_a, const int* swap_b,
                         int n_swaps);

/* Replay mode (off by default). on != 0: the next run records the device work of one pass, on all
 * its streams, into a HIP graph (stream capture; the completion events between operators become
 * edges of that graph) and launches it; later runs launch the recorded graph again instead of
 * issuing every operator. One recording is kept per binding of tensor vertices to storage, so
 * iterations that alternate between two bindings through purine_graph_swap_storage record twice
 * and replay from then on; adding a vertex or setting a stream discards the recordings. A pass is
 * replayed only if it is all device work on streams the graph created itself and neither timing
 * nor serial mode is on; otherwise the run issues its operators directly, as with replay off.
 * Results are bit-identical either way. Operator arguments are read when a pass is recorded:
 * change nothing behind the graph's back (contents of tensors may change freely, addresses and
 * attributes may not). on == 0 discards the recordings. */
int purine_graph_set_replay(purine_graph* g, int on);

/* What validation planned for the runs to come (both need a validated graph, PURINE_E_GRAPH
 * otherwise; the order the dispatcher fires in depends on the graph alone, section 2.1).
 * purine_graph_issue_plan: that firing order; writes up to cap operator ids, returns their number.
 * purine_graph_op_waits: the producers whose completion operator op_id will wait for before it is
 * issued: events on other streams for a device operator, on the host for a host operator.
 * Producers on the operator's own stream are ordered by the stream, and a producer is left out
 * when waiting for another one already implies it (a later operator of the same stream, or a wait
 * made by an earlier operator of the consumer's stream). An operator nobody waits for records no
 * event. Writes up to cap ids, returns their number; PURINE_E_ARG for a bad id. */
int purine_graph_issue_plan(const purine_graph* g, int* op_ids, int cap);
int purine_graph_op_waits(const purine_graph* g, int op_id, int* producer_ids, int cap);

/* Firing order of the last run: writes up to cap operator ids, returns how many operators fired. */
int purine_graph_fire_log(const purine_graph* g, int* op_ids, int cap);
int purine_graph_num_ops(const purine_graph* g);
int purine_graph_num_tensors(const purine_graph* g);

/* Per-operator device timing. With timing on, purine_graph_run brackets the main kernel of every
 * device operator with a pair of HIP events on the operator's own stream (the small second-pass
 * kernels of the split reductions are outside the bracket). After the run,
 * purine_graph_op_elapsed_ms gives the elapsed time of that bracket in the last run.
 * PURINE_E_ARG for a bad id, a host operator, or when the last run was not timed. */
int purine_graph_enable_timing(purine_graph* g, int on);
/* Timing on, but only operator op_id is bracketed (two event records per run instead of two per
 * operator, so the measurement does not perturb the run it measures). That operator also gets the
 * device to itself: its stream first waits for everything already issued on the graph's other
 * streams, and they wait for it, so the bracket measures the kernel alone. */
int purine_graph_time_only(purine_graph* g, int op_id);
/* on != 0: every operator runs with the device to itself (its stream waits for everything issued
 * before it on the graph's other streams, and they wait for it): kernels never overlap, whatever
 * their thread ids. Results are unchanged; meant for per-operator measurements. */
int purine_graph_set_serial(purine_graph* g, int on);
int purine_graph_op_elapsed_ms(purine_graph* g, int op_id, float* ms);

/* The same bracket for direct operator calls: the next operator call made by this host thread
 * records start_event (a hipEvent_t) just before its main kernel and stop_event just after it, on
 * the stream it was given, and then forgets the pair. Pass NULLs to cancel. */
void purine_set_kernel_probe(void* start_event, void* stop_event);

/* Tuning hook (host only, process-wide, not thread safe): forces the (rows, pixels) tile of the
 * forward / backward-data kernels to one of 128x128, 96x256, 96x128, 64x256, 128x64, 64x128, 32x256,
 * 64x64, 32x128; any other pair (e.g. 0, 0) restores the automatic choice. Results are bit-identical
 * for every shape: the reduction order per output element does not depend on it.
 * (48|16, 256|128) does the same for the 16-row-granular tiles of GEMMs with at most 16 or 33..48
 * rows, (192, 128) selects an uncalibrated tile.
 * For 1x1 / stride-1 / unpadded layers, which run the streaming GEMM kernel instead: (32|64|96, 2),
 * (64|96, 1) or (32|64, 4) force its rows per workgroup and pixels per lane, and (-1, anything) sends
 * those layers through the general kernel.
 * (anything, -1) makes every kernel take ordinary global loads with explicit zero fill instead of
 * range-checked raw buffer loads (the path tensors of 2 GiB and more take anyway). */
void purine_debug_force_tile(int bm, int bn);

/* Test hook (host only): n / d computed with the multiply-and-shift reciprocal that the kernels'
 * index arithmetic uses; valid for 0 <= n < 2^31 and 1 <= d < 2^31. */
uint32_t purine_debug_fastdiv(uint32_t n, uint32_t d);

#ifdef __cplusplus
}
#endif
#endif /* PURINE_H */

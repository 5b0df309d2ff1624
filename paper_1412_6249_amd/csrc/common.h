// Internal declarations shared by the host entry points and the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "purine.h"

namespace purine {

// Division of 0 <= n < 2^31 by a divisor fixed on the host, done with one high multiply, one masked
// add and a shift, with no branch (round-up reciprocal: m = ceil(2^(32+s)/d) with
// s = ceil(log2 d) - 1 fits 32 bits, and the error term n*e/2^(32+s) stays below 1/d for every
// n < 2^31; d = 1 has no such m, so it takes q = (0 + n) >> 0 through the add mask).
struct FastDiv {
    uint32_t m, s, add;
};

inline FastDiv make_fastdiv(uint32_t d) {
    FastDiv f{0u, 0u, 0xffffffffu};
    if (d <= 1) return f;
    uint32_t l = 0;
    while ((1ull << l) < d) ++l;           // l = ceil(log2 d) >= 1
    f.s = l - 1;
    f.add = 0u;
    const unsigned __int128 one = 1;
    const unsigned __int128 num = one << (32 + f.s);
    f.m = (uint32_t)((num + d - 1) / d);
    return f;
}

__host__ __device__ inline uint32_t fastdiv(uint32_t n, const FastDiv& f) {
#if defined(__HIP_DEVICE_COMPILE__)
    return (__umulhi(n, f.m) + (n & f.add)) >> f.s;
#else
    return ((uint32_t)(((uint64_t)n * f.m) >> 32) + (n & f.add)) >> f.s;
#endif
}

// Problem description of the weight-gradient implicit GEMM:
//   partial[split][k][(c,r,s)] = sum over pixels (n,p,q) of the split of dy[n,k,p,q] * x[n,c,p*sh-ph+r,q*sw-pw+s]
struct WgradParams {
    const void* x;
    const void* dy;
    float* out;        // partial sums [splits][K][CRS], or dw itself when splits == 1 and beta == 0
    int N, C, H, W, K, P, Q, R, S, sh, sw, ph, pw;
    int PQ, M, CRS, RS, HW;
    FastDiv div_pq, div_q, div_rs, div_s;
    int chunk;         // pixels per split, a multiple of the slab depth
    int tiles_i, tiles_j, splits;
    int c_tiles;       // per-tap column mode: channel tiles per tap (tiles_j = R*S*c_tiles)
    int x_ns, dy_ns;   // elements between consecutive images of x and of dy
    unsigned x_bytes, dy_bytes;   // tensor spans when the kernels may read them as raw buffers, else 0
    float* db_out;     // fused bias gradient: partial sums [splits][K], or null
};


struct ConvGeom {
    int N, C, H, W, K, R, S, P, Q, sh, sw, ph, pw;
    // elements between consecutive images of the x-shaped tensors (x, dx, the ReLU mask of dx) and
    // of the y-shaped ones (y, dy): C*H*W and K*P*Q unless the tensor is a channel-slice view
    int x_ns, y_ns;
};

// Launch plan of the forward / backward-data implicit GEMM: same answer for the workspace query and
// for the launch.
struct PixPlan {
    int mode;          // 0 forward, 1 backward-data with unit stride, 2 backward-data phase-folded
    bool flat;         // forward with fewer than 16 input channels: flattened (c,r,s) reduction, no scratch
    int bm, bn, tiles_i, tiles_pix;
    int Co, Ci;        // GEMM rows and gathered channels
    int Rt, St;        // taps of the reduction
    int Ci_pad, i_pad; // extents of the repacked filter A[Rt*St][Ci_pad][i_pad]
    size_t ws_bytes;   // scratch: repacked filter, then (bf16 tap kernels) the channels-blocked input copy
    size_t blk_offset; // byte offset of that copy inside the scratch (0: none)
    bool patch;        // bf16: the kernel that stages the input patch in LDS runs (no blocked copy)
    // 1x1 / stride 1 / unpadded layers: streaming GEMM kernel (used when the pointers are aligned
    // to gemm_tn elements; the fields above stay valid for the general kernel otherwise)
    bool gemm1x1;
    int gemm_tm, gemm_tn, gemm_tiles_i, gemm_tiles_pix;
    // ... with a split reduction when its tiles alone would leave most of the chip idle (the
    // fully-connected backward-data shape: few rows, few pixels, a long reduction)
    int gemm_splits, gemm_split_ci;
    size_t gemm_part_offset;   // byte offset of the fp32 partial tiles inside the scratch
};
PixPlan plan_conv_pix(const ConvGeom& g, bool bwd_data, int dtype, bool fused, bool accumulate = false);
void force_pix_tile(int bm, int bn);
bool patch_split_roles_forced();     // test hook: (-5, anything) gives it layers of few tiles too
bool patch_split_roles_disabled();   // tuning hook: (-4, anything) keeps the bf16 patch kernel on its one-role form
bool buffer_loads_disabled();   // tuning hook: (anything, -1) given to force_pix_tile

// Split of the pixel reduction of the weight gradient: same answer for the workspace query and
// for the launch.
struct WgradPlan {
    bool rows;         // bf16 3x3 layers: the row-staging kernel (one partial tile per persistent workgroup)
    bool cols;         // bf16 layers with C*R*S <= 160: whole-filter tiles per wavefront (conv_wgrad_cols_bf16.hip)
    bool taps;         // bf16 layers with C*R <= 32 and a known filter row shape: one tile per column tap (conv_wgrad_taps_bf16.hip)
    bool tap;          // columns are the channels of one tap (C >= 64) instead of flattened (c,r,s)
    int c_tiles;
    int bm, bn;        // tile extents along k and along the columns
    int tiles_i, tiles_j, splits, chunk;
    size_t ws_bytes;      // weight-gradient partials
    size_t db_ws_bytes;   // bias-gradient partials of the fused operator, placed behind them
};
WgradPlan plan_wgrad(const ConvGeom& g, int dtype);
bool wgrad_rows_bf16_applies(const ConvGeom& g, int* workers);
hipError_t launch_wgrad_rows_bf16(const ConvGeom& g, int workers, const void* x, const void* dy, float* partials,
                                  float* db_partials, hipStream_t st);
bool wgrad_taps_bf16_applies(const ConvGeom& g, int* workers);
hipError_t launch_wgrad_taps_bf16(const ConvGeom& g, const void* x, const void* dy, float* partials,
                                  float* db_partials, hipStream_t st);
bool wgrad_cols_bf16_applies(const ConvGeom& g, int* workers);
hipError_t launch_wgrad_cols_bf16(const ConvGeom& g, const void* x, const void* dy, float* partials,
                                  float* db_partials, hipStream_t st);
inline size_t wgrad_db_offset(const WgradPlan& pl) { return (pl.ws_bytes + 255) & ~(size_t)255; }

struct BiasBwdPlan {
    int parts;         // image groups per channel
    int imgs_per_part;
    size_t ws_bytes;
};
BiasBwdPlan plan_bias_bwd(int N, int K, int PQ);

// Maps a HIP status to a purine status and remembers the HIP error for purine_last_hip_error().
int hip_status(hipError_t e);

// One-shot event pair that brackets the main kernel of the next operator call of this host thread.
struct KernelProbe { hipEvent_t start, stop; };
KernelProbe take_kernel_probe();   // returns the pending pair (or NULLs) and clears it
struct ProbeScope {                 // records start on construction and stop on destruction
    KernelProbe p; hipStream_t st;
    explicit ProbeScope(hipStream_t s) : p(take_kernel_probe()), st(s) { if (p.start) (void)hipEventRecord(p.start, st); }
    // armed = false: an inert scope (the pending pair is left for an inner scope to take)
    ProbeScope(hipStream_t s, bool armed) : p(armed ? take_kernel_probe() : KernelProbe{nullptr, nullptr}), st(s) {
        if (p.start) (void)hipEventRecord(p.start, st);
    }
    ~ProbeScope() { if (p.stop) (void)hipEventRecord(p.stop, st); }
};

// Kernel launchers (defined in the .hip files). Each returns a hipError_t from the launch.
// Optional fused epilogue of the forward / backward-data kernels.
struct PixEpilogue {
    const void* bias = nullptr;   // forward: y = conv + bias[k]
    int relu = 0;                 // forward: y = max(y, 0)
    const void* mask = nullptr;   // backward-data: dx = mask > 0 ? dx : 0 (mask has dx's extents)
};
hipError_t launch_conv_pix(int dtype, const ConvGeom& g, const PixPlan& plan, const void* in,
                           const void* wt, void* out, float beta, void* ws, const PixEpilogue& epi,
                           hipStream_t st);
// db != null: also db = beta*db + sum of dy over pixels (fused BiasBwd), scratch behind dw's partials
hipError_t launch_conv_wgrad(int dtype, const ConvGeom& g, const WgradPlan& plan, const void* x,
                             const void* dy, float* dw, float* db, float beta, void* ws, hipStream_t st);
hipError_t launch_bias_fwd(int dtype, const void* b, void* y, int N, int K, int PQ, hipStream_t st);
hipError_t launch_bias_bwd(int dtype, const void* dy, float* db, float beta, int N, int K, int PQ,
                           const BiasBwdPlan& plan, void* ws, hipStream_t st);
hipError_t launch_relu_fwd(int dtype, const void* x, void* y, int64_t n, hipStream_t st);
hipError_t launch_relu_bwd(int dtype, const void* x, const void* dy, void* dx, int64_t n,
                           hipStream_t st);
hipError_t launch_bias_rows(const float* b, float* y, int N, int K, hipStream_t st);
hipError_t launch_fc_finish_bf16(const float* acc, const void* b, void* y, int N, int K, hipStream_t st);
// bf16 fully-connected data gradient: scratch bytes and slicing (SIZE_MAX: rows are not whole
// 16-byte packets, the kernel does not apply)
size_t fc_dgrad_bf16_plan(int64_t N, int64_t C, int64_t K, int* slices, int* k_per_slice);
hipError_t launch_fc_dgrad_bf16(const void* dy, const void* w, void* dx, int N, int K, int C, void* ws, hipStream_t st);
// db[k] = beta*db[k] + sum_n dy[n][k] for a dense [N][K] matrix (fixed summation order)
hipError_t launch_fc_bias_bwd(int dtype, const void* dy, float* db, int N, int K, float beta, hipStream_t st);
// out0 = in0^T and out1 = in1^T for dense 2-byte matrices of `rows` x cols0 / cols1 elements, one launch
hipError_t launch_transpose16_pair(const void* in0, void* out0, int cols0, const void* in1, void* out1, int cols1, int rows,
                                   hipStream_t st);
// bf16 fully-connected weight gradient on the transposed matrices (batches of a multiple of 8 samples)
bool fc_wgrad_bf16_applies(int64_t N, int64_t C, int64_t K);
hipError_t launch_fc_wgrad_bf16(const void* dyT, const void* xT, float* dw, int N, int K, int C, bool accumulate,
                                hipStream_t st);
hipError_t launch_relu_view(int dtype, bool bwd, const void* x, const void* dy, void* out, int N, int run,
                            int64_t x_ns, int64_t dy_ns, int64_t out_ns, hipStream_t st);
hipError_t launch_sgd_update(int dtype, const void* w, const float* dw, void* new_w, float lr,
                             int64_t n, hipStream_t st);
hipError_t launch_maxpool_fwd(int dtype, const void* x, void* y, int32_t* arg, int NC, int H, int W,
                              int P, int Q, int k, int stride, int pad, hipStream_t st);
hipError_t launch_maxpool_bwd(int dtype, const void* dy, const int32_t* arg, void* dx, const void* y, float beta,
                              int NC, int H, int W, int P, int Q, int k, int stride, int pad,
                              hipStream_t st);
hipError_t launch_copy_channels(int dtype, const void* src, void* dst, int N, int c_count,
                                int src_C, int src_c0, int dst_C, int dst_c0, int HW,
                                hipStream_t st);
hipError_t launch_sum(int dtype, const void* const* terms, int n_terms, void* out, int64_t n,
                      hipStream_t st);

}  // namespace purine

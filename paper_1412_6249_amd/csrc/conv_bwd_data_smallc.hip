// Backward-data for layers with very few input channels (C <= 4: the first layer of a CNN).
//
// With C = 3 the output side of the backward-data GEMM is 3 rows tall, so a 32-row MFMA tile would
// idle 90% of the matrix pipe, and with stride > 1 only 1/(sh*sw) of the (r,s) taps touch a given
// input position. fp32 vector FMA has the same peak rate as fp32 MFMA on this chip, so this case
// runs on the vector ALUs instead:
//   - a thread owns SW consecutive input columns w = wq*SW + b - pw (b = 0..SW-1) of one row h and
//     all C channels; the wavefront's lanes run along wq, rows of one phase a = (h+ph) mod sh;
//   - only the taps that can hit are visited: r = a + sh*r', s = b + SW*s' (phase decomposition of
//     the strided transposed convolution), so no multiply is wasted on structural zeros;
//   - one dy value is loaded per (k, r', s') and reused for all C*SW (channel, column-phase) FMAs;
//   - r, s, k and the row phase are uniform across the wavefront, so the filter taps are scalar
//     operands.
// Stores are SW consecutive floats per lane, i.e. fully coalesced.
#include "common.h"

namespace purine {
namespace {

template <typename T> __device__ __forceinline__ float ldv(const T* p, int i);
template <> __device__ __forceinline__ float ldv<float>(const float* p, int i) { return p[i]; }
template <> __device__ __forceinline__ float ldv<uint16_t>(const uint16_t* p, int i) {
    return __uint_as_float(((uint32_t)p[i]) << 16);
}
template <typename T> __device__ __forceinline__ void stv(T* p, int i, float v);
template <> __device__ __forceinline__ void stv<float>(float* p, int i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void stv<uint16_t>(uint16_t* p, int i, float v) {
    uint32_t u = __float_as_uint(v);
    uint32_t r = u + 0x7FFFu + ((u >> 16) & 1u);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) r = 0x7FC00000u;
    p[i] = (uint16_t)(r >> 16);
}

struct SmallCParams {
    const void* dy; const void* wt; void* dx;
    int N, C, H, W, K, P, Q, R, S, sh, ph, pw;
    int wq_min, Wq;            // column groups: wq = wq_min .. wq_min + Wq - 1
    FastDiv div_wq;
    float beta;
};

template <typename T, int C, int SW>
__global__ __launch_bounds__(256) void bwd_data_smallc_kernel(const SmallCParams p) {
    const T* __restrict__ dy = (const T*)p.dy;
    const T* __restrict__ wt = (const T*)p.wt;
    T* __restrict__ dx = (T*)p.dx;

    const int n = blockIdx.y / p.sh;
    const int a = blockIdx.y - n * p.sh;                 // row phase: (h + ph) mod sh == a
    // rows of this phase: h = hq*sh + a - ph, 0 <= h < H
    const int t = p.ph - a;
    const int hq_min = t > 0 ? (t + p.sh - 1) / p.sh : 0;
    const int top = p.H - 1 + p.ph - a;
    const int hq_max = top >= 0 ? top / p.sh : -1;       // no row of this phase when top < 0
    const int Hq = hq_max - hq_min + 1;

    const int idx = blockIdx.x * 256 + threadIdx.x;
    const int hqi = fastdiv(idx, p.div_wq);
    const int wqi = idx - hqi * p.Wq;
    const bool live = hqi < Hq;
    const int hq = hq_min + hqi;
    const int wq = p.wq_min + wqi;
    const int h = hq * p.sh + a - p.ph;

    float acc[C][SW];
#pragma unroll
    for (int c = 0; c < C; ++c)
#pragma unroll
        for (int b = 0; b < SW; ++b) acc[c][b] = 0.0f;

    const int RS = p.R * p.S;
    const int ns = (p.S + SW - 1) / SW;
    const int dy_img = n * p.K * p.P * p.Q;
    for (int k = 0; k < p.K; ++k) {
        const int dy_plane = dy_img + k * p.P * p.Q;
        const int w_k = k * C * RS;
        for (int r = a, rp = 0; r < p.R; r += p.sh, ++rp) {
            const int pp = hq - rp;
            const bool row_ok = live && (unsigned)pp < (unsigned)p.P;
            const int w_kr = w_k + r * p.S;
            for (int sp = 0; sp < ns; ++sp) {
                const int qq = wq - sp;
                const bool ok = row_ok && (unsigned)qq < (unsigned)p.Q;
                const float v = ok ? ldv<T>(dy, dy_plane + pp * p.Q + qq) : 0.0f;
#pragma unroll
                for (int b = 0; b < SW; ++b) {
                    const int s = b + SW * sp;
                    if (s < p.S) {
#pragma unroll
                        for (int c = 0; c < C; ++c)
                            acc[c][b] = fmaf(v, ldv<T>(wt, w_kr + c * RS + s), acc[c][b]);
                    }
                }
            }
        }
    }
    if (!live) return;
#pragma unroll
    for (int c = 0; c < C; ++c) {
        const int row = ((n * C + c) * p.H + h) * p.W;
#pragma unroll
        for (int b = 0; b < SW; ++b) {
            const int w = wq * SW + b - p.pw;
            if ((unsigned)w < (unsigned)p.W) {
                float v = acc[c][b];
                if (p.beta != 0.0f) v += ldv<T>(dx, row + w);
                stv<T>(dx, row + w, v);
            }
        }
    }
}

template <typename T, int C, int SW>
hipError_t launch_one(SmallCParams& p, int max_hq, hipStream_t st) {
    const long long per_plane = (long long)max_hq * p.Wq;
    dim3 grid((unsigned)((per_plane + 255) / 256), (unsigned)(p.N * p.sh));
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    hipLaunchKernelGGL((bwd_data_smallc_kernel<T, C, SW>), grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

template <typename T, int C>
hipError_t by_sw(SmallCParams& p, int sw, int max_hq, hipStream_t st) {
    switch (sw) {
        case 1: return launch_one<T, C, 1>(p, max_hq, st);
        case 2: return launch_one<T, C, 2>(p, max_hq, st);
        case 3: return launch_one<T, C, 3>(p, max_hq, st);
        case 4: return launch_one<T, C, 4>(p, max_hq, st);
        default: return hipErrorInvalidValue;
    }
}

template <typename T>
hipError_t by_c(SmallCParams& p, int sw, int max_hq, hipStream_t st) {
    switch (p.C) {
        case 1: return by_sw<T, 1>(p, sw, max_hq, st);
        case 2: return by_sw<T, 2>(p, sw, max_hq, st);
        case 3: return by_sw<T, 3>(p, sw, max_hq, st);
        case 4: return by_sw<T, 4>(p, sw, max_hq, st);
        default: return hipErrorInvalidValue;
    }
}

}  // namespace

bool conv_bwd_data_smallc_applies(const ConvGeom& g) {
    // grid.y = N*sh must fit 65535; C and the column stride are template parameters
    return g.C <= 4 && g.sw <= 4 && (long long)g.N * g.sh <= 65535;
}

hipError_t launch_conv_bwd_data_smallc(int dtype, const ConvGeom& g, const void* dy, const void* wt,
                                       void* dx, float beta, hipStream_t st) {
    SmallCParams p{};
    p.dy = dy; p.wt = wt; p.dx = dx;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q;
    p.R = g.R; p.S = g.S; p.sh = g.sh; p.ph = g.ph; p.pw = g.pw;
    p.wq_min = g.pw / g.sw;
    const int wq_max = (g.W - 1 + g.pw) / g.sw;
    p.Wq = wq_max - p.wq_min + 1;
    p.div_wq = make_fastdiv(p.Wq);
    p.beta = beta;
    // the tallest row phase has ceil(H / sh) rows (one more when the phases straddle the padding)
    const int max_hq = (g.H + g.sh - 1) / g.sh + 1;
    if (dtype == PURINE_F32) return by_c<float>(p, g.sw, max_hq, st);
    return by_c<uint16_t>(p, g.sw, max_hq, st);
}

}  // namespace purine

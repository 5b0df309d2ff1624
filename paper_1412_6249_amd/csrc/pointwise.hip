// HBM-bound operators: Bias / BiasBwd of the convolution layer (paper Figure 1(b)) and the exact
// support operators (ReLU, max-pool, channel copy, fan-in sum) that chain layers together.
// All of them stream each tensor once with coalesced accesses; none uses atomics.
#include "common.h"
#include <type_traits>

namespace purine {
namespace {

__device__ __forceinline__ float bf2f(uint16_t b) { return __uint_as_float(((uint32_t)b) << 16); }
__device__ __forceinline__ uint16_t f2bf(float v) {
    uint32_t u = __float_as_uint(v);
    uint32_t r = u + 0x7FFFu + ((u >> 16) & 1u);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) r = 0x7FC00000u;
    return (uint16_t)(r >> 16);
}
template <typename T> __device__ __forceinline__ float ldf(const T* p, size_t i);
template <> __device__ __forceinline__ float ldf<float>(const float* p, size_t i) { return p[i]; }
template <> __device__ __forceinline__ float ldf<uint16_t>(const uint16_t* p, size_t i) { return bf2f(p[i]); }
template <typename T> __device__ __forceinline__ void stf(T* p, size_t i, float v);
template <> __device__ __forceinline__ void stf<float>(float* p, size_t i, float v) { p[i] = v; }
template <> __device__ __forceinline__ void stf<uint16_t>(uint16_t* p, size_t i, float v) { p[i] = f2bf(v); }

constexpr int TPB = 256;

// 16-byte packets: 4 floats or 8 bfloat16. The vector kernels below move one packet per lane
// (1 KiB per wavefront instruction); the scalar forms handle rows whose length or start is not a
// multiple of a packet.
template <typename T> struct Pk;
template <> struct Pk<float> {
    static constexpr int N = 4;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[4]) {
        f[0] = __uint_as_float(v.x); f[1] = __uint_as_float(v.y);
        f[2] = __uint_as_float(v.z); f[3] = __uint_as_float(v.w);
    }
    static __device__ __forceinline__ uint4 pack(const float (&f)[4]) {
        return make_uint4(__float_as_uint(f[0]), __float_as_uint(f[1]), __float_as_uint(f[2]), __float_as_uint(f[3]));
    }
};
template <> struct Pk<uint16_t> {
    static constexpr int N = 8;
    static __device__ __forceinline__ void unpack(const uint4& v, float (&f)[8]) {
        const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            f[2 * i] = __uint_as_float(w[i] << 16);
            f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    }
    static __device__ __forceinline__ uint4 pack(const float (&f)[8]) {
        uint32_t w[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) w[i] = (uint32_t)f2bf(f[2 * i]) | ((uint32_t)f2bf(f[2 * i + 1]) << 16);
        return make_uint4(w[0], w[1], w[2], w[3]);
    }
};

// ---- Bias: y[n,k,:,:] += b[k]; grid.x = plane (n*K + k), grid.y = chunks of the plane ------------
template <typename T, bool VEC>
__global__ __launch_bounds__(TPB) void bias_fwd_kernel(const T* __restrict__ b, T* __restrict__ y,
                                                       int K, int PQ) {
    const int plane = blockIdx.x;
    const float bv = ldf<T>(b, plane % K);
    T* row = y + (size_t)plane * PQ;
    if (VEC) {
        constexpr int V = Pk<T>::N;
        uint4* r4 = reinterpret_cast<uint4*>(row);
        for (int i = blockIdx.y * TPB + threadIdx.x; i < PQ / V; i += gridDim.y * TPB) {
            float f[V];
            Pk<T>::unpack(r4[i], f);
#pragma unroll
            for (int e = 0; e < V; ++e) f[e] += bv;
            r4[i] = Pk<T>::pack(f);
        }
    } else {
        for (int i = blockIdx.y * TPB + threadIdx.x; i < PQ; i += gridDim.y * TPB)
            stf<T>(row, i, ldf<T>(row, i) + bv);
    }
}

// ---- BiasBwd: lane -> wavefront (shuffle) -> workgroup (LDS) partial per (k, image group),
//      then one thread per channel adds the group partials in order -------------------------------
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_down(v, off, 64);
    return v;
}

template <typename T, bool VEC>
__global__ __launch_bounds__(TPB) void bias_bwd_partial_kernel(const T* __restrict__ dy,
                                                               float* __restrict__ partial, int N,
                                                               int K, int PQ, int imgs_per_part,
                                                               int parts) {
    const int k = blockIdx.x, part = blockIdx.y;
    const int n0 = part * imgs_per_part;
    const int n1 = min(N, n0 + imgs_per_part);
    float acc = 0.0f;
    for (int n = n0; n < n1; ++n) {
        const T* row = dy + ((size_t)n * K + k) * PQ;
        if (VEC) {
            constexpr int V = Pk<T>::N;
            const uint4* r4 = reinterpret_cast<const uint4*>(row);
            for (int i = threadIdx.x; i < PQ / V; i += TPB) {
                float f[V];
                Pk<T>::unpack(r4[i], f);
#pragma unroll
                for (int e = 0; e < V; ++e) acc += f[e];
            }
        } else {
            for (int i = threadIdx.x; i < PQ; i += TPB) acc += ldf<T>(row, i);
        }
    }
    __shared__ float wsum[TPB / 64];
    acc = wave_sum(acc);
    if ((threadIdx.x & 63) == 0) wsum[threadIdx.x >> 6] = acc;
    __syncthreads();
    if (threadIdx.x == 0) {
        float t = 0.0f;
#pragma unroll
        for (int w = 0; w < TPB / 64; ++w) t += wsum[w];
        partial[(size_t)k * parts + part] = t;
    }
}

__global__ __launch_bounds__(TPB) void bias_bwd_final_kernel(const float* __restrict__ partial,
                                                             float* __restrict__ db, int K,
                                                             int parts, float beta) {
    const int k = blockIdx.x * TPB + threadIdx.x;
    if (k >= K) return;
    float acc = beta != 0.0f ? db[k] : 0.0f;
    for (int i = 0; i < parts; ++i) acc += partial[(size_t)k * parts + i];
    db[k] = acc;
}

// ---- ReLU: packets for the bulk, scalars for the tail ------------------------------------------
template <typename T>
__global__ __launch_bounds__(TPB) void relu_fwd_kernel(const T* x, T* y, size_t n) {
    constexpr int V = Pk<T>::N;
    const size_t nv = n / V, stride = (size_t)gridDim.x * TPB, t0 = (size_t)blockIdx.x * TPB + threadIdx.x;
    const uint4* x4 = reinterpret_cast<const uint4*>(x);
    uint4* y4 = reinterpret_cast<uint4*>(y);
    for (size_t i = t0; i < nv; i += stride) {
        float f[V];
        Pk<T>::unpack(x4[i], f);
#pragma unroll
        for (int e = 0; e < V; ++e) f[e] = f[e] > 0.0f ? f[e] : 0.0f;
        y4[i] = Pk<T>::pack(f);
    }
    for (size_t i = nv * V + t0; i < n; i += stride) {
        const float v = ldf<T>(x, i);
        stf<T>(y, i, v > 0.0f ? v : 0.0f);
    }
}
// ReLU and its gradient on channel-slice views: grid.y = image, each image a dense run of `run`
// elements at its own distance between images. VEC: run and the distances are whole 16-byte packets.
template <typename T, bool BWD, bool VEC>
__global__ __launch_bounds__(TPB) void relu_view_kernel(const T* x, const T* dy, T* out,
                                                        int run, size_t x_ns, size_t dy_ns, size_t out_ns) {
    const size_t n = blockIdx.y;
    const T* xi = x + n * x_ns;
    const T* gi = BWD ? dy + n * dy_ns : nullptr;
    T* oi = out + n * out_ns;
    const int t0 = blockIdx.x * TPB + threadIdx.x, stride = gridDim.x * TPB;
    if (VEC) {
        constexpr int V = Pk<T>::N;
        for (int i = t0; i < run / V; i += stride) {
            float v[V], g[V];
            Pk<T>::unpack(reinterpret_cast<const uint4*>(xi)[i], v);
            if (BWD) Pk<T>::unpack(reinterpret_cast<const uint4*>(gi)[i], g);
#pragma unroll
            for (int e = 0; e < V; ++e) g[e] = v[e] > 0.0f ? (BWD ? g[e] : v[e]) : 0.0f;
            reinterpret_cast<uint4*>(oi)[i] = Pk<T>::pack(g);
        }
    } else {
        for (int i = t0; i < run; i += stride) {
            const float v = ldf<T>(xi, i);
            stf<T>(oi, i, v > 0.0f ? (BWD ? ldf<T>(gi, i) : v) : 0.0f);
        }
    }
}

// ---- bias of a fully-connected layer: y[n][k] += b[k] on a dense [N][K] fp32 matrix --------------
__global__ __launch_bounds__(TPB) void bias_rows_kernel(const float* __restrict__ b, float* y, int K, size_t n) {
    const size_t stride = (size_t)gridDim.x * TPB;
    for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < n; i += stride) y[i] += b[i % (size_t)K];
}

// Bias gradient of a fully-connected layer: db[k] = beta*db[k] + sum_n dy[n][k] on a dense [N][K]
// matrix. 64 columns per workgroup (a wavefront reads whole rows of them); wavefront g adds the rows
// n = g, g + 4, ... in four interleaved chains, and the four partial sums are added in wavefront
// order: a fixed order, the same result on every run.
template <typename T>
__global__ __launch_bounds__(256) void fc_bias_bwd_kernel(const T* __restrict__ dy, float* db, int N, int K, float beta) {
    __shared__ float part[4][64];
    const int lane = threadIdx.x & 63, g = threadIdx.x >> 6, k = (int)blockIdx.x * 64 + lane;
    float s[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (k < K) {
        int n = g;
        for (; n + 12 < N; n += 16) {
#pragma unroll
            for (int j = 0; j < 4; ++j) s[j] += ldf<T>(dy, (size_t)(n + 4 * j) * K + k);
        }
        for (int j = 0; n < N; n += 4, ++j) s[j] += ldf<T>(dy, (size_t)n * K + k);
    }
    part[g][lane] = (s[0] + s[1]) + (s[2] + s[3]);
    __syncthreads();
    if (g == 0 && k < K) {
        const float t = ((part[0][lane] + part[1][lane]) + part[2][lane]) + part[3][lane];
        db[k] = beta != 0.0f ? db[k] + t : t;
    }
}

// bf16 fully-connected forward, last step: y[n][k] = bf16(acc[n][k] + b[k]) from the fp32 product
// matrix (one rounding, to nearest even, after the bias is added in fp32). b may be null.
__global__ __launch_bounds__(TPB) void fc_finish_bf16_kernel(const float* __restrict__ acc, const uint16_t* __restrict__ b,
                                                             uint16_t* __restrict__ y, int K, size_t n) {
    const size_t stride = (size_t)gridDim.x * TPB;
    for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < n; i += stride)
        y[i] = f2bf(acc[i] + (b ? bf2f(b[i % (size_t)K]) : 0.0f));
}

// out[c][r] = in[r][c] for two dense 2-byte matrices of `rows` x cols0 and `rows` x cols1 elements in
// one launch (the first tiles0 workgroups take the first matrix); 64x64 tiles through LDS (row pitch
// 66 elements: a tile column read walks through different banks)
__global__ __launch_bounds__(256) void transpose16_pair_kernel(const uint16_t* __restrict__ in0, uint16_t* __restrict__ out0,
                                                               int cols0, unsigned tiles0, const uint16_t* __restrict__ in1,
                                                               uint16_t* __restrict__ out1, int cols1, int rows) {
    __shared__ uint16_t tile[64][66];
    const bool second = blockIdx.x >= tiles0;
    const uint16_t* __restrict__ in = second ? in1 : in0;
    uint16_t* __restrict__ out = second ? out1 : out0;
    const int cols = second ? cols1 : cols0;
    const unsigned b = second ? blockIdx.x - tiles0 : blockIdx.x;
    const int tiles_c = (cols + 63) / 64;
    const int r0 = (int)(b / tiles_c) * 64, c0 = (int)(b % tiles_c) * 64;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int j = ty; j < 64; j += 4) {
        const int r = r0 + j, c = c0 + tx;
        tile[j][tx] = (r < rows && c < cols) ? in[(size_t)r * cols + c] : (uint16_t)0;
    }
    __syncthreads();
    for (int j = ty; j < 64; j += 4) {
        const int c = c0 + j, r = r0 + tx;
        if (c < cols && r < rows) out[(size_t)c * rows + r] = tile[tx][j];
    }
}

// ---- SGD update: new_w = w - lr * dw (one fused multiply-add in fp32 per element) ---------------
// Packets of the parameter tensor (4 floats or 8 bfloat16) against 4-float packets of the fp32
// gradient. new_w may be w itself: every element is read before it is written by the same lane.
template <typename T>
__global__ __launch_bounds__(TPB) void sgd_update_kernel(const T* w, const float* __restrict__ dw,
                                                         T* nw, float lr, size_t n) {
    constexpr int V = Pk<T>::N;
    const size_t nv = n / V, stride = (size_t)gridDim.x * TPB, t0 = (size_t)blockIdx.x * TPB + threadIdx.x;
    const uint4* w4 = reinterpret_cast<const uint4*>(w);
    const float4* g4 = reinterpret_cast<const float4*>(dw);
    uint4* o4 = reinterpret_cast<uint4*>(nw);
    for (size_t i = t0; i < nv; i += stride) {
        float f[V];
        Pk<T>::unpack(w4[i], f);
#pragma unroll
        for (int q = 0; q < V / 4; ++q) {
            const float4 g = g4[i * (V / 4) + q];
            f[4 * q + 0] = fmaf(-lr, g.x, f[4 * q + 0]);
            f[4 * q + 1] = fmaf(-lr, g.y, f[4 * q + 1]);
            f[4 * q + 2] = fmaf(-lr, g.z, f[4 * q + 2]);
            f[4 * q + 3] = fmaf(-lr, g.w, f[4 * q + 3]);
        }
        o4[i] = Pk<T>::pack(f);
    }
    for (size_t i = nv * V + t0; i < n; i += stride) stf<T>(nw, i, fmaf(-lr, dw[i], ldf<T>(w, i)));
}

template <typename T>
__global__ __launch_bounds__(TPB) void relu_bwd_kernel(const T* __restrict__ x, const T* dy, T* dx,
                                                       size_t n) {
    constexpr int V = Pk<T>::N;
    const size_t nv = n / V, stride = (size_t)gridDim.x * TPB, t0 = (size_t)blockIdx.x * TPB + threadIdx.x;
    const uint4* x4 = reinterpret_cast<const uint4*>(x);
    const uint4* g4 = reinterpret_cast<const uint4*>(dy);
    uint4* o4 = reinterpret_cast<uint4*>(dx);
    for (size_t i = t0; i < nv; i += stride) {
        float f[V], g[V];
        Pk<T>::unpack(x4[i], f);
        Pk<T>::unpack(g4[i], g);
#pragma unroll
        for (int e = 0; e < V; ++e) g[e] = f[e] > 0.0f ? g[e] : 0.0f;
        o4[i] = Pk<T>::pack(g);
    }
    for (size_t i = nv * V + t0; i < n; i += stride) {
        const float v = ldf<T>(x, i);
        stf<T>(dx, i, v > 0.0f ? ldf<T>(dy, i) : 0.0f);
    }
}

// ---- max pooling --------------------------------------------------------------------------------
// Work is cut into runs of consecutive planes: a workgroup owns POOL_CHUNK consecutive elements of a
// group of `ppw` planes (grid.x: group, grid.y: chunk) (small planes are batched so that every workgroup has a few thousand
// elements; large planes are split). Outputs are written in memory order (coalesced); the window
// reads overlap between neighbours and are served by L1. Index arithmetic uses the reciprocal
// division; window size and stride are template constants for the common shapes (K = 0: runtime).
constexpr int POOL_CHUNK = 2048;

struct PoolParams {
    int NC, H, W, P, Q, HW, PQ, k, stride, pad, ppw;
    FastDiv div_pq, div_q, div_hw, div_w;
    float beta;
};

template <typename T, int K, int S>
__global__ __launch_bounds__(TPB) void maxpool_fwd_kernel(const T* __restrict__ x, T* __restrict__ y,
                                                          int32_t* __restrict__ arg, const PoolParams pp) {
    const int k = K ? K : pp.k, st = K ? S : pp.stride;
    const int lim = min(pp.ppw * pp.PQ, ((int)blockIdx.y + 1) * POOL_CHUNK);
    for (int l = blockIdx.y * POOL_CHUNK + threadIdx.x; l < lim; l += TPB) {
        const int pl = fastdiv(l, pp.div_pq);
        const int o = l - pl * pp.PQ;
        const int nc = blockIdx.x * pp.ppw + pl;
        if (nc >= pp.NC) break;
        const int p = fastdiv(o, pp.div_q), q = o - p * pp.Q;
        const int h0 = p * st - pp.pad, w0 = q * st - pp.pad;
        const T* plane = x + (size_t)nc * pp.HW;
        int best = -1;
        float bv = 0.0f;
        if (K) {
#pragma unroll
            for (int r = 0; r < (K ? K : 1); ++r)
#pragma unroll
                for (int c = 0; c < (K ? K : 1); ++c) {
                    const int h = h0 + r, w = w0 + c;
                    const bool ok = ((unsigned)h < (unsigned)pp.H) & ((unsigned)w < (unsigned)pp.W);
                    const int at = ok ? h * pp.W + w : 0;          // clamped, branch-free
                    const float v = ldf<T>(plane, at);
                    const bool take = ok & ((best < 0) | (v > bv));
                    best = take ? at : best;
                    bv = take ? v : bv;
                }
        } else {
            for (int r = 0; r < k; ++r) {
                const int h = h0 + r;
                if ((unsigned)h >= (unsigned)pp.H) continue;
                for (int c = 0; c < k; ++c) {
                    const int w = w0 + c;
                    if ((unsigned)w >= (unsigned)pp.W) continue;
                    const float v = ldf<T>(plane, (size_t)h * pp.W + w);
                    if (best < 0 || v > bv) { best = h * pp.W + w; bv = v; }
                }
            }
        }
        const size_t out = (size_t)nc * pp.PQ + o;
        stf<T>(y, out, bv);
        arg[out] = best;
    }
}

// Gather form of the pooling gradient: each input position visits the windows that cover it in
// row-major (p,q) order and adds dy where that window's winner is this position. `y` (may be
// null): the pooling output of the forward pass; windows whose winner was not positive pass no
// gradient. When the pooled tensor is a ReLU output that is its ReLU gradient (a position that won
// a window holds that window's y), which would otherwise be a pass of its own over dx.
template <typename T, int K, int S>
__global__ __launch_bounds__(TPB) void maxpool_bwd_kernel(const T* __restrict__ dy,
                                                          const int32_t* __restrict__ arg,
                                                          T* dx, const T* __restrict__ y, const PoolParams pp) {
    const int k = K ? K : pp.k, st = K ? S : pp.stride;
    constexpr int NW = K ? (K + S - 1) / (S ? S : 1) : 1;   // windows per axis that can cover a position
    const int lim = min(pp.ppw * pp.HW, ((int)blockIdx.y + 1) * POOL_CHUNK);
    for (int l = blockIdx.y * POOL_CHUNK + threadIdx.x; l < lim; l += TPB) {
        const int pl = fastdiv(l, pp.div_hw);
        const int e = l - pl * pp.HW;
        const int nc = blockIdx.x * pp.ppw + pl;
        if (nc >= pp.NC) break;
        const int h = fastdiv(e, pp.div_w), w = e - h * pp.W;
        // windows p with p*stride - pad <= h <= p*stride - pad + k - 1
        const int p_hi = min(pp.P - 1, (h + pp.pad) / st);
        const int q_hi = min(pp.Q - 1, (w + pp.pad) / st);
        int p_lo = h + pp.pad - k + 1;
        p_lo = p_lo <= 0 ? 0 : (p_lo + st - 1) / st;
        int q_lo = w + pp.pad - k + 1;
        q_lo = q_lo <= 0 ? 0 : (q_lo + st - 1) / st;
        const size_t obase = (size_t)nc * pp.PQ;
        const size_t at = (size_t)nc * pp.HW + e;
        const float old = pp.beta != 0.0f ? ldf<T>(dx, at) : 0.0f;
        float acc = old;
        if (K) {
#pragma unroll
            for (int a = 0; a < NW; ++a)
#pragma unroll
                for (int b = 0; b < NW; ++b) {
                    const int p = p_lo + a, q = q_lo + b;
                    const bool in = (p <= p_hi) & (q <= q_hi);
                    const int o = in ? p * pp.Q + q : 0;           // clamped, branch-free
                    const bool hit = in & (arg[obase + o] == e) & (!y || ldf<T>(y, obase + o) > 0.0f);
                    const float g = ldf<T>(dy, obase + o);
                    acc += hit ? g : 0.0f;
                }
        } else {
            for (int p = p_lo; p <= p_hi; ++p)
                for (int q = q_lo; q <= q_hi; ++q) {
                    const size_t o = obase + p * pp.Q + q;
                    if (arg[o] == e && (!y || ldf<T>(y, o) > 0.0f)) acc += ldf<T>(dy, o);
                }
        }
        stf<T>(dx, at, acc);
    }
}

// The same with the windows' winners and gradients staged in LDS: a workgroup owns whole planes (a few
// thousand input positions in all), copies their arg and dy planes into LDS with coalesced loads
// (one {winner, gradient} pair per window, so a look-up is one 8-byte read), and every position
// then looks its up-to-NW x NW windows up there. What goes to and comes from global memory is one
// coalesced pass per tensor (in the kernel above every position's gathers of arg and dy go through
// the caches, and the kernel runs at half the rate of a copy). Same windows in the same order:
// bit-identical results. quads != 0 (a workgroup's first position is a multiple of four positions
// from an aligned dx): a thread takes four consecutive positions, decodes the first and steps to
// the others, and dx moves as packets of four.
template <typename T, int K, int S>
__global__ __launch_bounds__(TPB) void maxpool_bwd_staged_kernel(const T* __restrict__ dy,
                                                                 const int32_t* __restrict__ arg,
                                                                 T* dx, const T* __restrict__ y, const PoolParams pp,
                                                                 const int quads) {
    extern __shared__ __attribute__((aligned(16))) unsigned char pool_smem[];
    int2* win_s = reinterpret_cast<int2*>(pool_smem);                 // [ppw][PQ] {winner, gradient bits}
    const int k = K ? K : pp.k, st = K ? S : pp.stride;
    constexpr int NW = K ? (K + S - 1) / (S ? S : 1) : 1;
    const int nc0 = blockIdx.x * pp.ppw;
    const int planes = min(pp.ppw, pp.NC - nc0);
    {
        const size_t base = (size_t)nc0 * pp.PQ;
        const int n = planes * pp.PQ;
        for (int i = threadIdx.x; i < n; i += TPB) {
            // the gradient of a window whose winner was not positive is dropped here, once per window
            const float g = (!y || ldf<T>(y, base + i) > 0.0f) ? ldf<T>(dy, base + i) : 0.0f;
            win_s[i] = make_int2(arg[base + i], __float_as_int(g));
        }
    }
    __syncthreads();
    // beta*dx + the gradients of the windows that chose position e = (h, w) of the workgroup's plane pl
    auto gather = [&](int pl, int e, int h, int w, float old) -> float {
        const int p_hi = min(pp.P - 1, (h + pp.pad) / st);
        const int q_hi = min(pp.Q - 1, (w + pp.pad) / st);
        int p_lo = h + pp.pad - k + 1;
        p_lo = p_lo <= 0 ? 0 : (p_lo + st - 1) / st;
        int q_lo = w + pp.pad - k + 1;
        q_lo = q_lo <= 0 ? 0 : (q_lo + st - 1) / st;
        const int obase = pl * pp.PQ;
        float acc = old;
        if (K) {
#pragma unroll
            for (int a = 0; a < NW; ++a)
#pragma unroll
                for (int b = 0; b < NW; ++b) {
                    const int p = p_lo + a, q = q_lo + b;
                    const bool in = (p <= p_hi) & (q <= q_hi);
                    const int2 win = win_s[obase + (in ? p * pp.Q + q : 0)];   // clamped, branch-free
                    acc += (in & (win.x == e)) ? __int_as_float(win.y) : 0.0f;
                }
        } else {
            for (int p = p_lo; p <= p_hi; ++p)
                for (int q = q_lo; q <= q_hi; ++q) {
                    const int2 win = win_s[obase + p * pp.Q + q];
                    if (win.x == e) acc += __int_as_float(win.y);
                }
        }
        return acc;
    };
    const int lim = planes * pp.HW;
    const size_t first = (size_t)nc0 * pp.HW;
    int done = 0;
    if (quads) {
        typedef typename std::conditional<sizeof(T) == 4, float4, ushort4>::type Quad;
        const int nq = lim >> 2;
        for (int j = threadIdx.x; j < nq; j += TPB) {
            const int l = j * 4;
            int pl = fastdiv(l, pp.div_hw);
            int e = l - pl * pp.HW;
            int h = fastdiv(e, pp.div_w), w = e - h * pp.W;
            Quad* at = reinterpret_cast<Quad*>(dx + first + l);
            float v[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            if (pp.beta != 0.0f) {
                const Quad o = *at;
                if constexpr (sizeof(T) == 4) { v[0] = o.x; v[1] = o.y; v[2] = o.z; v[3] = o.w; }
                else { v[0] = bf2f(o.x); v[1] = bf2f(o.y); v[2] = bf2f(o.z); v[3] = bf2f(o.w); }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                v[i] = gather(pl, e, h, w, v[i]);
                ++e; ++w;
                if (w == pp.W) { w = 0; ++h; }
                if (e == pp.HW) { e = 0; h = 0; ++pl; }
            }
            Quad o;
            if constexpr (sizeof(T) == 4) { o.x = v[0]; o.y = v[1]; o.z = v[2]; o.w = v[3]; }
            else { o.x = f2bf(v[0]); o.y = f2bf(v[1]); o.z = f2bf(v[2]); o.w = f2bf(v[3]); }
            *at = o;
        }
        done = nq * 4;
    }
    for (int l = done + threadIdx.x; l < lim; l += TPB) {
        const int pl = fastdiv(l, pp.div_hw);
        const int e = l - pl * pp.HW;
        const int h = fastdiv(e, pp.div_w), w = e - h * pp.W;
        const float old = pp.beta != 0.0f ? ldf<T>(dx, first + l) : 0.0f;
        stf<T>(dx, first + l, gather(pl, e, h, w, old));
    }
}

// ---- 3x3 / stride 1 / pad 1 pooling on fp32 planes whose width is a multiple of 4 ----------------
// (the pooling branch of an inception module). A lane owns four consecutive positions of one row:
// per window row it needs the aligned packet of those four columns plus the column on either side,
// so 3 packets + 6 scalars replace 36 scalar loads, and the outputs leave as packets. Winners and
// sums are taken in the same order as in the general kernels (bit-identical results).
struct Pool3Params {
    int NC, H, W, HW, W4;      // W4 = W / 4 packets per row
    FastDiv div_row4, div_w4;  // by H * W4 (packets per plane) and by W4
    long long total4;          // packets in all
    float beta;
};

__global__ __launch_bounds__(TPB) void maxpool3_fwd_vec_kernel(const float* __restrict__ x, float* __restrict__ y,
                                                               int32_t* __restrict__ arg, const Pool3Params pp) {
    for (long long i = (long long)blockIdx.x * TPB + threadIdx.x; i < pp.total4; i += (long long)gridDim.x * TPB) {
        // plane index and packet inside the plane (the host keeps the packet count below 2^31)
        const int per_plane = pp.H * pp.W4;
        const int nc = fastdiv((uint32_t)i, pp.div_row4);
        const int r4 = (int)i - nc * per_plane;
        const int p = fastdiv(r4, pp.div_w4);
        const int q0 = (r4 - p * pp.W4) * 4;
        const float* plane = x + (size_t)nc * pp.HW;
        float bv[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        int best[4] = {-1, -1, -1, -1};
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int h = p - 1 + r;
            const bool row_ok = (unsigned)h < (unsigned)pp.H;
            const int hb = (row_ok ? h : p) * pp.W;                 // clamped row: values unused when !row_ok
            const float4 v4 = *reinterpret_cast<const float4*>(plane + hb + q0);
            const bool l_ok = row_ok & (q0 > 0), r_ok = row_ok & (q0 + 4 < pp.W);
            const float vl = plane[hb + (q0 > 0 ? q0 - 1 : q0)];
            const float vr = plane[hb + (q0 + 4 < pp.W ? q0 + 4 : q0)];
            const float v[6] = {vl, v4.x, v4.y, v4.z, v4.w, vr};
            const bool ok[6] = {l_ok, row_ok, row_ok, row_ok, row_ok, r_ok};
#pragma unroll
            for (int o = 0; o < 4; ++o)
#pragma unroll
                for (int c = 0; c < 3; ++c) {                       // window column c of output o is v[o + c]
                    const bool take = ok[o + c] & ((best[o] < 0) | (v[o + c] > bv[o]));
                    best[o] = take ? h * pp.W + q0 + o + c - 1 : best[o];
                    bv[o] = take ? v[o + c] : bv[o];
                }
        }
        const size_t out = (size_t)nc * pp.HW + (size_t)p * pp.W + q0;
        *reinterpret_cast<float4*>(y + out) = make_float4(bv[0], bv[1], bv[2], bv[3]);
        *reinterpret_cast<int4*>(arg + out) = make_int4(best[0], best[1], best[2], best[3]);
    }
}

__global__ __launch_bounds__(TPB) void maxpool3_bwd_vec_kernel(const float* __restrict__ dy,
                                                               const int32_t* __restrict__ arg, float* dx,
                                                               const Pool3Params pp) {
    for (long long i = (long long)blockIdx.x * TPB + threadIdx.x; i < pp.total4; i += (long long)gridDim.x * TPB) {
        const int per_plane = pp.H * pp.W4;
        const int nc = fastdiv((uint32_t)i, pp.div_row4);
        const int r4 = (int)i - nc * per_plane;
        const int h = fastdiv(r4, pp.div_w4);
        const int w0 = (r4 - h * pp.W4) * 4;
        const size_t base = (size_t)nc * pp.HW;
        const size_t at = base + (size_t)h * pp.W + w0;
        float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (pp.beta != 0.0f) {
            const float4 o = *reinterpret_cast<const float4*>(dx + at);
            acc[0] = o.x; acc[1] = o.y; acc[2] = o.z; acc[3] = o.w;
        }
        // windows (p, q) with p in h-1..h+1 and q in w-1..w+1 cover position (h, w); visited in (p, q) order
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            const int p = h - 1 + r;
            const bool row_ok = (unsigned)p < (unsigned)pp.H;
            const size_t rb = base + (size_t)(row_ok ? p : h) * pp.W;
            const float4 g4 = *reinterpret_cast<const float4*>(dy + rb + w0);
            const int4 a4 = *reinterpret_cast<const int4*>(arg + rb + w0);
            const int li = w0 > 0 ? w0 - 1 : w0, ri = w0 + 4 < pp.W ? w0 + 4 : w0;
            const bool l_ok = row_ok & (w0 > 0), r_ok = row_ok & (w0 + 4 < pp.W);
            const float g[6] = {dy[rb + li], g4.x, g4.y, g4.z, g4.w, dy[rb + ri]};
            const int a[6] = {arg[rb + li], a4.x, a4.y, a4.z, a4.w, arg[rb + ri]};
            const bool ok[6] = {l_ok, row_ok, row_ok, row_ok, row_ok, r_ok};
#pragma unroll
            for (int o = 0; o < 4; ++o) {
                const int e = h * pp.W + w0 + o;                    // this position's index in its plane
#pragma unroll
                for (int c = 0; c < 3; ++c) {
                    const bool hit = ok[o + c] & (a[o + c] == e);
                    acc[o] += hit ? g[o + c] : 0.0f;
                }
            }
        }
        *reinterpret_cast<float4*>(dx + at) = make_float4(acc[0], acc[1], acc[2], acc[3]);
    }
}

// ---- channel-slice copy (concat and its inverse) -------------------------------------------------
template <typename T, bool VEC>
__global__ __launch_bounds__(TPB) void copy_channels_kernel(const T* __restrict__ src,
                                                            T* __restrict__ dst, int c_count,
                                                            int src_C, int src_c0, int dst_C,
                                                            int dst_c0, int HW) {
    const int n = blockIdx.y;
    const size_t run = (size_t)c_count * HW;   // the slice of one image is contiguous on both sides
    const T* s = src + ((size_t)n * src_C + src_c0) * HW;
    T* d = dst + ((size_t)n * dst_C + dst_c0) * HW;
    if (VEC) {   // HW is a multiple of a packet, so every slice starts and ends on a packet
        const uint4* s4 = reinterpret_cast<const uint4*>(s);
        uint4* d4 = reinterpret_cast<uint4*>(d);
        const size_t nv = run / Pk<T>::N;
        for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < nv; i += (size_t)gridDim.x * TPB)
            d4[i] = s4[i];
    } else {
        for (size_t i = (size_t)blockIdx.x * TPB + threadIdx.x; i < run; i += (size_t)gridDim.x * TPB)
            d[i] = s[i];
    }
}

// ---- fan-in sum ------------------------------------------------------------------------------------
struct SumArgs { const void* t[8]; int n; };
template <typename T>
__global__ __launch_bounds__(TPB) void sum_kernel(SumArgs a, T* out, size_t n) {
    constexpr int V = Pk<T>::N;
    const size_t nv = n / V, stride = (size_t)gridDim.x * TPB, t0 = (size_t)blockIdx.x * TPB + threadIdx.x;
    for (size_t i = t0; i < nv; i += stride) {
        float acc[V];
        Pk<T>::unpack(reinterpret_cast<const uint4*>(a.t[0])[i], acc);
        for (int j = 1; j < a.n; ++j) {
            float f[V];
            Pk<T>::unpack(reinterpret_cast<const uint4*>(a.t[j])[i], f);
#pragma unroll
            for (int e = 0; e < V; ++e) acc[e] += f[e];
        }
        reinterpret_cast<uint4*>(out)[i] = Pk<T>::pack(acc);
    }
    for (size_t i = nv * V + t0; i < n; i += stride) {
        float acc = ldf<T>((const T*)a.t[0], i);
        for (int j = 1; j < a.n; ++j) acc += ldf<T>((const T*)a.t[j], i);
        stf<T>(out, i, acc);
    }
}

inline unsigned blocks_for(size_t n, unsigned cap = 256 * 16) {
    size_t b = (n + TPB - 1) / TPB;
    if (b < 1) b = 1;
    return (unsigned)(b > cap ? cap : b);
}

}  // namespace

BiasBwdPlan plan_bias_bwd(int N, int K, int PQ) {
    BiasBwdPlan pl{};
    (void)PQ;
    // about 2048 workgroups in total, at least one image per group
    int parts = (2048 + K - 1) / K;
    if (parts > N) parts = N;
    if (parts < 1) parts = 1;
    pl.imgs_per_part = (N + parts - 1) / parts;
    pl.parts = (N + pl.imgs_per_part - 1) / pl.imgs_per_part;
    pl.ws_bytes = (size_t)K * pl.parts * sizeof(float);
    return pl;
}

#define BY_DTYPE(dtype, CALL_F32, CALL_BF16) \
    do { if ((dtype) == PURINE_F32) { CALL_F32; } else { CALL_BF16; } } while (0)

hipError_t launch_bias_fwd(int dtype, const void* b, void* y, int N, int K, int PQ, hipStream_t st) {
    const int V = dtype == PURINE_F32 ? 4 : 8;
    const bool vec = PQ % V == 0;
    dim3 grid((unsigned)(N * K), blocks_for(vec ? PQ / V : PQ, 64));
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    if (vec)
        BY_DTYPE(dtype,
                 hipLaunchKernelGGL((bias_fwd_kernel<float, true>), grid, dim3(TPB), 0, st, (const float*)b, (float*)y, K, PQ),
                 hipLaunchKernelGGL((bias_fwd_kernel<uint16_t, true>), grid, dim3(TPB), 0, st, (const uint16_t*)b, (uint16_t*)y, K, PQ));
    else
        BY_DTYPE(dtype,
                 hipLaunchKernelGGL((bias_fwd_kernel<float, false>), grid, dim3(TPB), 0, st, (const float*)b, (float*)y, K, PQ),
                 hipLaunchKernelGGL((bias_fwd_kernel<uint16_t, false>), grid, dim3(TPB), 0, st, (const uint16_t*)b, (uint16_t*)y, K, PQ));
    return hipGetLastError();
}

hipError_t launch_bias_bwd(int dtype, const void* dy, float* db, float beta, int N, int K, int PQ,
                           const BiasBwdPlan& plan, void* ws, hipStream_t st) {
    dim3 grid((unsigned)K, (unsigned)plan.parts);
    float* partial = (float*)ws;
    {
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    if (PQ % (dtype == PURINE_F32 ? 4 : 8) == 0)
        BY_DTYPE(dtype,
                 hipLaunchKernelGGL((bias_bwd_partial_kernel<float, true>), grid, dim3(TPB), 0, st, (const float*)dy, partial, N, K, PQ, plan.imgs_per_part, plan.parts),
                 hipLaunchKernelGGL((bias_bwd_partial_kernel<uint16_t, true>), grid, dim3(TPB), 0, st, (const uint16_t*)dy, partial, N, K, PQ, plan.imgs_per_part, plan.parts));
    else
        BY_DTYPE(dtype,
                 hipLaunchKernelGGL((bias_bwd_partial_kernel<float, false>), grid, dim3(TPB), 0, st, (const float*)dy, partial, N, K, PQ, plan.imgs_per_part, plan.parts),
                 hipLaunchKernelGGL((bias_bwd_partial_kernel<uint16_t, false>), grid, dim3(TPB), 0, st, (const uint16_t*)dy, partial, N, K, PQ, plan.imgs_per_part, plan.parts));
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(bias_bwd_final_kernel, dim3((K + TPB - 1) / TPB), dim3(TPB), 0, st,
                       (const float*)partial, db, K, plan.parts, beta);
    return hipGetLastError();
}

hipError_t launch_relu_fwd(int dtype, const void* x, void* y, int64_t n, hipStream_t st) {
    dim3 grid(blocks_for((size_t)n / 4 + 1));
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    BY_DTYPE(dtype,
             hipLaunchKernelGGL(relu_fwd_kernel<float>, grid, dim3(TPB), 0, st, (const float*)x, (float*)y, (size_t)n),
             hipLaunchKernelGGL(relu_fwd_kernel<uint16_t>, grid, dim3(TPB), 0, st, (const uint16_t*)x, (uint16_t*)y, (size_t)n));
    return hipGetLastError();
}

hipError_t launch_bias_rows(const float* b, float* y, int N, int K, hipStream_t st) {
    const size_t n = (size_t)N * K;
    (void)hipGetLastError();
    hipLaunchKernelGGL(bias_rows_kernel, dim3(blocks_for(n)), dim3(TPB), 0, st, b, y, K, n);
    return hipGetLastError();
}

hipError_t launch_fc_finish_bf16(const float* acc, const void* b, void* y, int N, int K, hipStream_t st) {
    const size_t n = (size_t)N * K;
    (void)hipGetLastError();
    hipLaunchKernelGGL(fc_finish_bf16_kernel, dim3(blocks_for(n)), dim3(TPB), 0, st, acc, (const uint16_t*)b,
                       (uint16_t*)y, K, n);
    return hipGetLastError();
}

hipError_t launch_fc_bias_bwd(int dtype, const void* dy, float* db, int N, int K, float beta, hipStream_t st) {
    if (N < 1 || K < 1) return hipErrorInvalidValue;
    const dim3 grid((unsigned)((K + 63) / 64));
    (void)hipGetLastError();
    if (dtype == PURINE_BF16)
        hipLaunchKernelGGL(fc_bias_bwd_kernel<uint16_t>, grid, dim3(256), 0, st, (const uint16_t*)dy, db, N, K, beta);
    else
        hipLaunchKernelGGL(fc_bias_bwd_kernel<float>, grid, dim3(256), 0, st, (const float*)dy, db, N, K, beta);
    return hipGetLastError();
}

hipError_t launch_transpose16_pair(const void* in0, void* out0, int cols0, const void* in1, void* out1, int cols1, int rows,
                                   hipStream_t st) {
    if (rows < 1 || cols0 < 1 || cols1 < 1) return hipErrorInvalidValue;
    const long long row_tiles = (rows + 63) / 64;
    const long long tiles0 = row_tiles * ((cols0 + 63) / 64), tiles1 = row_tiles * ((cols1 + 63) / 64);
    if (tiles0 + tiles1 > 0x7fffffffLL) return hipErrorInvalidValue;
    (void)hipGetLastError();
    hipLaunchKernelGGL(transpose16_pair_kernel, dim3((unsigned)(tiles0 + tiles1)), dim3(256), 0, st, (const uint16_t*)in0,
                       (uint16_t*)out0, cols0, (unsigned)tiles0, (const uint16_t*)in1, (uint16_t*)out1, cols1, rows);
    return hipGetLastError();
}

hipError_t launch_relu_view(int dtype, bool bwd, const void* x, const void* dy, void* out, int N, int run,
                            int64_t x_ns, int64_t dy_ns, int64_t out_ns, hipStream_t st) {
    const int V = dtype == PURINE_BF16 ? 8 : 4;
    const bool vec = run % V == 0 && x_ns % V == 0 && dy_ns % V == 0 && out_ns % V == 0;
    dim3 grid(blocks_for((size_t)(vec ? run / V : run), 64), (unsigned)N);
    if (N > 65535) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
#define RV(T, B, V) hipLaunchKernelGGL((relu_view_kernel<T, B, V>), grid, dim3(TPB), 0, st, (const T*)x, (const T*)dy, \
                                       (T*)out, run, (size_t)x_ns, (size_t)dy_ns, (size_t)out_ns)
#define RV2(T) do { if (bwd) { if (vec) RV(T, true, true); else RV(T, true, false); }                     \
                    else     { if (vec) RV(T, false, true); else RV(T, false, false); } } while (0)
    if (dtype == PURINE_BF16) RV2(uint16_t); else RV2(float);
#undef RV2
#undef RV
    return hipGetLastError();
}

hipError_t launch_sgd_update(int dtype, const void* w, const float* dw, void* new_w, float lr,
                             int64_t n, hipStream_t st) {
    dim3 grid(blocks_for((size_t)n / 4 + 1));
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    BY_DTYPE(dtype,
             hipLaunchKernelGGL(sgd_update_kernel<float>, grid, dim3(TPB), 0, st, (const float*)w, dw, (float*)new_w, lr, (size_t)n),
             hipLaunchKernelGGL(sgd_update_kernel<uint16_t>, grid, dim3(TPB), 0, st, (const uint16_t*)w, dw, (uint16_t*)new_w, lr, (size_t)n));
    return hipGetLastError();
}

hipError_t launch_relu_bwd(int dtype, const void* x, const void* dy, void* dx, int64_t n,
                           hipStream_t st) {
    dim3 grid(blocks_for((size_t)n / 4 + 1));
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    BY_DTYPE(dtype,
             hipLaunchKernelGGL(relu_bwd_kernel<float>, grid, dim3(TPB), 0, st, (const float*)x, (const float*)dy, (float*)dx, (size_t)n),
             hipLaunchKernelGGL(relu_bwd_kernel<uint16_t>, grid, dim3(TPB), 0, st, (const uint16_t*)x, (const uint16_t*)dy, (uint16_t*)dx, (size_t)n));
    return hipGetLastError();
}

namespace {
PoolParams pool_params(int NC, int H, int W, int P, int Q, int k, int stride, int pad, int per_plane, float beta) {
    PoolParams pp{};
    pp.NC = NC; pp.H = H; pp.W = W; pp.P = P; pp.Q = Q; pp.HW = H * W; pp.PQ = P * Q;
    pp.k = k; pp.stride = stride; pp.pad = pad; pp.beta = beta;
    pp.ppw = per_plane >= POOL_CHUNK ? 1 : POOL_CHUNK / per_plane;
    if (pp.ppw > NC) pp.ppw = NC;
    pp.div_pq = make_fastdiv(pp.PQ); pp.div_q = make_fastdiv(Q);
    pp.div_hw = make_fastdiv(pp.HW); pp.div_w = make_fastdiv(W);
    return pp;
}
dim3 pool_grid(const PoolParams& pp, int per_plane) {
    const long long per_group = (long long)pp.ppw * per_plane;
    // x: plane groups (up to 2^31 - 1), y: chunks of one group (up to 65535)
    return dim3((unsigned)((pp.NC + pp.ppw - 1) / pp.ppw), (unsigned)((per_group + POOL_CHUNK - 1) / POOL_CHUNK));
}
// the packet kernels: fp32, 3x3 / stride 1 / pad 1 (output extents = input extents), rows of whole packets
bool pool3_vec_applies(int dtype, int NC, int H, int W, int P, int Q, int k, int stride, int pad, const void* a,
                       const void* b, const void* c) {
    return dtype == PURINE_F32 && k == 3 && stride == 1 && pad == 1 && P == H && Q == W && W % 4 == 0 &&
           (long long)NC * H * (W / 4) < 0x7fffffffLL &&
           (((uintptr_t)a | (uintptr_t)b | (uintptr_t)c) & 15u) == 0;
}
Pool3Params pool3_params(int NC, int H, int W, float beta) {
    Pool3Params p{};
    p.NC = NC; p.H = H; p.W = W; p.HW = H * W; p.W4 = W / 4;
    p.div_w4 = make_fastdiv(p.W4);
    p.div_row4 = make_fastdiv(H * p.W4);
    p.total4 = (long long)NC * H * p.W4;
    p.beta = beta;
    return p;
}
#define POOL_SHAPES(CALL)                                           \
    if (k == 3 && stride == 1) { CALL(3, 1); }                      \
    else if (k == 3 && stride == 2) { CALL(3, 2); }                 \
    else if (k == 2 && stride == 2) { CALL(2, 2); }                 \
    else { CALL(0, 0); }
}  // namespace

hipError_t launch_maxpool_fwd(int dtype, const void* x, void* y, int32_t* arg, int NC, int H, int W,
                              int P, int Q, int k, int stride, int pad, hipStream_t st) {
    // a group of planes is indexed with 32-bit arithmetic; groups go to grid.y
    if ((long long)H * W > 0x3fffffffLL || (long long)P * Q > 0x3fffffffLL) return hipErrorInvalidValue;
    if (pool3_vec_applies(dtype, NC, H, W, P, Q, k, stride, pad, x, y, arg)) {
        const Pool3Params p3 = pool3_params(NC, H, W, 0.0f);
        ProbeScope probe(st);
        (void)hipGetLastError();
        hipLaunchKernelGGL(maxpool3_fwd_vec_kernel, dim3(blocks_for((size_t)p3.total4)), dim3(TPB), 0, st,
                           (const float*)x, (float*)y, arg, p3);
        return hipGetLastError();
    }
    const PoolParams pp = pool_params(NC, H, W, P, Q, k, stride, pad, P * Q, 0.0f);
    const dim3 grid = pool_grid(pp, P * Q);
    if (grid.y > 65535u) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
#define CALL(K, S)                                                                                              \
    BY_DTYPE(dtype,                                                                                             \
             hipLaunchKernelGGL((maxpool_fwd_kernel<float, K, S>), grid, dim3(TPB), 0, st, (const float*)x, (float*)y, arg, pp),       \
             hipLaunchKernelGGL((maxpool_fwd_kernel<uint16_t, K, S>), grid, dim3(TPB), 0, st, (const uint16_t*)x, (uint16_t*)y, arg, pp))
    POOL_SHAPES(CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_maxpool_bwd(int dtype, const void* dy, const int32_t* arg, void* dx, const void* y, float beta,
                              int NC, int H, int W, int P, int Q, int k, int stride, int pad,
                              hipStream_t st) {
    if ((long long)H * W > 0x3fffffffLL || (long long)P * Q > 0x3fffffffLL) return hipErrorInvalidValue;
    if (!y && pool3_vec_applies(dtype, NC, H, W, P, Q, k, stride, pad, dy, dx, arg)) {
        const Pool3Params p3 = pool3_params(NC, H, W, beta);
        ProbeScope probe(st);
        (void)hipGetLastError();
        hipLaunchKernelGGL(maxpool3_bwd_vec_kernel, dim3(blocks_for((size_t)p3.total4)), dim3(TPB), 0, st,
                           (const float*)dy, arg, (float*)dx, p3);
        return hipGetLastError();
    }
    PoolParams pp = pool_params(NC, H, W, P, Q, k, stride, pad, H * W, beta);
    // Whole planes per workgroup with their arg and dy planes in LDS: up to about 8K positions per
    // workgroup, a multiple of four planes (then every workgroup starts a multiple of four positions
    // into dx and dx moves as packets), when 8 bytes per window of those planes fit 48 KB and the
    // workgroup has at most 16K positions to walk.
    {
        long long ppw = 8192 / ((long long)H * W);
        if (ppw > NC / 2048) ppw = NC / 2048;         // at least 2048 workgroups, eight per CU
        if (ppw >= 4) ppw = ppw / 4 * 4;
        else if (4LL * H * W <= 16384) ppw = 4;
        else if (ppw < 1) ppw = 1;
        if (ppw > NC) ppw = NC;
        if (ppw * P * Q * 8 <= 48 * 1024 && ppw * H * W <= 16384) {
            pp.ppw = (int)ppw;
            const unsigned groups = (unsigned)((NC + pp.ppw - 1) / pp.ppw);
            const size_t lds = (size_t)pp.ppw * P * Q * 8;
            const int elem = dtype == PURINE_BF16 ? 2 : 4;
            const int quads = ((ppw * H * W) % 4 == 0 || groups == 1) && ((uintptr_t)dx % (4 * elem)) == 0;
            ProbeScope probe(st);
            (void)hipGetLastError();
#define CALL(K, S)                                                                                              \
    BY_DTYPE(dtype,                                                                                             \
             hipLaunchKernelGGL((maxpool_bwd_staged_kernel<float, K, S>), dim3(groups), dim3(TPB), lds, st, (const float*)dy, arg, (float*)dx, (const float*)y, pp, quads),     \
             hipLaunchKernelGGL((maxpool_bwd_staged_kernel<uint16_t, K, S>), dim3(groups), dim3(TPB), lds, st, (const uint16_t*)dy, arg, (uint16_t*)dx, (const uint16_t*)y, pp, quads))
            POOL_SHAPES(CALL)
#undef CALL
            return hipGetLastError();
        }
    }
    const dim3 grid = pool_grid(pp, H * W);
    if (grid.y > 65535u) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
#define CALL(K, S)                                                                                              \
    BY_DTYPE(dtype,                                                                                             \
             hipLaunchKernelGGL((maxpool_bwd_kernel<float, K, S>), grid, dim3(TPB), 0, st, (const float*)dy, arg, (float*)dx, (const float*)y, pp),     \
             hipLaunchKernelGGL((maxpool_bwd_kernel<uint16_t, K, S>), grid, dim3(TPB), 0, st, (const uint16_t*)dy, arg, (uint16_t*)dx, (const uint16_t*)y, pp))
    POOL_SHAPES(CALL)
#undef CALL
    return hipGetLastError();
}

hipError_t launch_copy_channels(int dtype, const void* src, void* dst, int N, int c_count,
                                int src_C, int src_c0, int dst_C, int dst_c0, int HW,
                                hipStream_t st) {
    dim3 grid(blocks_for((size_t)c_count * HW, 256), (unsigned)N);
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    if (HW % (dtype == PURINE_F32 ? 4 : 8) == 0)
        BY_DTYPE(dtype,
                 hipLaunchKernelGGL((copy_channels_kernel<float, true>), grid, dim3(TPB), 0, st, (const float*)src, (float*)dst, c_count, src_C, src_c0, dst_C, dst_c0, HW),
                 hipLaunchKernelGGL((copy_channels_kernel<uint16_t, true>), grid, dim3(TPB), 0, st, (const uint16_t*)src, (uint16_t*)dst, c_count, src_C, src_c0, dst_C, dst_c0, HW));
    else
        BY_DTYPE(dtype,
                 hipLaunchKernelGGL((copy_channels_kernel<float, false>), grid, dim3(TPB), 0, st, (const float*)src, (float*)dst, c_count, src_C, src_c0, dst_C, dst_c0, HW),
                 hipLaunchKernelGGL((copy_channels_kernel<uint16_t, false>), grid, dim3(TPB), 0, st, (const uint16_t*)src, (uint16_t*)dst, c_count, src_C, src_c0, dst_C, dst_c0, HW));
    return hipGetLastError();
}

hipError_t launch_sum(int dtype, const void* const* terms, int n_terms, void* out, int64_t n,
                      hipStream_t st) {
    SumArgs a{};
    a.n = n_terms;
    for (int i = 0; i < n_terms; ++i) a.t[i] = terms[i];
    dim3 grid(blocks_for((size_t)n / 4 + 1));
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    BY_DTYPE(dtype,
             hipLaunchKernelGGL(sum_kernel<float>, grid, dim3(TPB), 0, st, a, (float*)out, (size_t)n),
             hipLaunchKernelGGL(sum_kernel<uint16_t>, grid, dim3(TPB), 0, st, a, (uint16_t*)out, (size_t)n));
    return hipGetLastError();
}

}  // namespace purine

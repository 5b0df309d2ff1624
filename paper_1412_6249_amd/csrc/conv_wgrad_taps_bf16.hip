// bf16 weight gradient for layers with at most 32 (channel, filter row) pairs, C*R <= 32, and a
// column stride of 1 or 2: the 7x7 / stride 2 first layer of an image network and its relatives
// (ConvBwdWeight of paper Figure 1(b)):
//
//     dw[k, c, r, s] = sum over (n, p, q) of dy[n, k, p, q] * x[n, c, sh*p - ph + r, sw*q - pw + s]
//
// A small output tile with a very long reduction that streams dy exactly once; the pass is bound by
// memory, so the kernel is built to keep many bytes in flight and to spend little LDS bandwidth:
//
//  * The MFMA columns are the (c, r) pairs; the S column taps of a filter row are S separate
//    accumulator tiles that share ONE read of the staged input row: the window of tap s is the
//    aligned 16-byte packet of the lane's row, shifted by floor((s - pw) / sw) elements, and is put
//    together in registers from the packet and the dword on either side (funnel shifts). The taps
//    are template parameters, so every shift is a compile-time constant.
//  * With a column stride of 2 the eight consecutive pixels of an operand read every second input
//    column: the input rows are de-interleaved on their way into LDS (a byte permute per packet),
//    one plane per column parity, so that a window is 8 consecutive elements of one plane.
//  * dy rows need no re-layout (8 consecutive pixels of one channel = one 16-byte packet).
//  * A workgroup of four wavefronts owns 64 output channels: wavefront = (32-channel half, parity of
//    the 16-pixel step). Workgroups are persistent over a contiguous range of (image, output row)
//    pairs, one output row per iteration: its dy row (64 channels) and the R input rows of every
//    channel come in as 16-byte packets in the order they lie in memory. The packets are requested
//    TWO iterations ahead (two register sets, used in turn) and stored into the other half of an
//    LDS double buffer one iteration ahead; one barrier per iteration; two workgroups per CU.
//
// Partial tiles go to scratch as [worker][k][c][r][s] (fp32) together with the bias-gradient
// partials of the fused operator; the fixed-order second pass of the general kernel adds them.
#include "common.h"

namespace purine {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned u32x2 __attribute__((ext_vector_type(2)));

constexpr int NT = 256;             // four wavefronts
constexpr int KT = 64;              // output channels per workgroup
// Element of a plane row that holds index 0 (left halo before it). Column stride 2: planes take
// 8-byte stores (four pixels of a parity), so index 0 may sit 8 bytes past a 16-byte boundary, which
// makes the 16 elements q - 4 .. q + 11 around a step's window two ALIGNED 16-byte reads; with
// stride 1 the planes take whole 16-byte packets and index 0 stays on a boundary.
constexpr int plane_org(int sw) { return sw == 2 ? 12 : 8; }
constexpr int X_ROUNDS = 3;         // 16-byte packets per thread and iteration, at most: input rows
constexpr int D_ROUNDS = 4;         // ... and the dy row

// LDS pitch: at least `bytes`, an odd number of 16-byte packets, so that 16-byte reads of 8
// consecutive rows fall into distinct bank groups
inline int odd16_pitch(int bytes) {
    int packets = (bytes + 15) / 16;
    if ((packets & 1) == 0) packets += 1;
    return packets * 16;
}

struct TapsWgradParams {
    const uint16_t* x; const uint16_t* dy; float* out; float* db_out;
    int N, C, H, W, K, P, Q, R, sh, ph;
    int x_ns, dy_ns;
    unsigned x_bytes, dy_bytes;
    int k_groups, workers;             // grid = workers * k_groups
    int rows_total, rows_per_worker;   // flattened (n, p) output rows
    int cr, ncol;                      // C*R, C*R*S
    int ppitch, dpitch;                // LDS bytes per plane row / per dy row
    int xchunks, dychunks;             // 16-byte packets per input row (W / 8) and dy row (Q / 8)
    int steps;                         // 16-pixel MFMA steps per output row: Q / 16
    int x_tasks, d_tasks;              // packets per iteration
    int d_bytes, spare_off, buf_bytes; // dy rows of a buffer; offset of its spare packets; whole buffer
    FastDiv div_p;
};

__device__ __forceinline__ float sum8(const u32x4 u) {
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += __uint_as_float(u[i] << 16) + __uint_as_float(u[i] & 0xffff0000u);
    return s;
}

// column tap s of a filter with S columns, left padding PW and column stride SW reads plane
// tap_plane (column parity) at element q + tap_shift
constexpr int tap_plane(int s, int PW, int SW) { return (((s - PW) % SW) + SW) % SW; }
constexpr int tap_shift(int s, int PW, int SW) { return ((s - PW) - tap_plane(s, PW, SW)) / SW; }

template <int S, int PW, int SW>
__global__ __launch_bounds__(NT, 2) void wgrad_taps_bf16_kernel(const TapsWgradParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // buffer b at smem + b * buf_bytes: dy rows [KT] of dpitch bytes, planes [SW][C*R] of ppitch bytes, spare packets

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int khalf = lane >> 5;
    const int kt = wave & 1, parity = wave >> 1;
    const int kg = blockIdx.x % p.k_groups, worker = blockIdx.x / p.k_groups;
    const int k0 = kg * KT;
    const int g0 = worker * p.rows_per_worker;
    const int g1 = min(g0 + p.rows_per_worker, p.rows_total);
    const int plane_bytes = p.cr * p.ppitch;

    // ---- once: zeros everywhere (halos of the planes, the channels past K)
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < 2 * p.buf_bytes / 16; i += NT) *reinterpret_cast<u32x4*>(smem + i * 16) = z;
    }

    // lanes past the last (c, r) pair repeat it; their columns are never stored
    constexpr int ORG = plane_org(SW);
    const int b_row = p.d_bytes + min(lane & 31, p.cr - 1) * p.ppitch + (ORG + khalf * 8) * 2;
    const int a_addr = (kt * 32 + (lane & 31)) * p.dpitch + khalf * 16;

    // ---- load tasks of this thread (fixed over the iterations). A thread without a task in a round
    // loads zeros (range check) and stores them into a spare packet of its own: no branch around loads
    // or stores in the loop, which lets the compiler wait for exactly the older register set.
    int x_g[X_ROUNDS], x_l[X_ROUNDS], x_r[X_ROUNDS];
#pragma unroll
    for (int j = 0; j < X_ROUNDS; ++j) {
        const int t = tid + j * NT;
        const int chunk = t % p.xchunks, row = t / p.xchunks;      // row = c * R + r
        const int c = row / p.R, r = row - c * p.R;
        const bool live = t < p.x_tasks;
        x_g[j] = live ? (c * p.H * p.W + chunk * 8) * 2 : -1;
        x_l[j] = live ? p.d_bytes + row * p.ppitch + (ORG + chunk * (8 / SW)) * 2 : p.spare_off + tid * 16;
        x_r[j] = r;
    }
    int d_g[D_ROUNDS], d_l[D_ROUNDS];
#pragma unroll
    for (int j = 0; j < D_ROUNDS; ++j) {
        const int t = tid + j * NT;
        const int chunk = t % p.dychunks, k = t / p.dychunks;
        const bool live = t < p.d_tasks;
        d_g[j] = (live && k0 + k < p.K) ? ((k0 + k) * p.P * p.Q + chunk * 8) * 2 : -1;
        d_l[j] = live ? k * p.dpitch + chunk * 16 : p.spare_off + tid * 16;
    }
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), (short)0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_dy =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.dy), (short)0, (int)p.dy_bytes, 0x00020000);
    u32x4 xr0[X_ROUNDS], dr0[D_ROUNDS], xr1[X_ROUNDS], dr1[D_ROUNDS];   // the two register sets

    // packets of flattened output row g (a row at or past g1, input rows outside the image and channels
    // past K come back as zeros: range-checked loads)
    auto load_iter = [&](int g, u32x4 (&xr)[X_ROUNDS], u32x4 (&dr)[D_ROUNDS]) {
        const bool ok = g < g1;
        const int n = fastdiv(g, p.div_p), pp = g - n * p.P;
        const int hb = p.sh * pp - p.ph;
        const int xb = n * p.x_ns * 2;
        const int db = n * p.dy_ns * 2 + pp * p.Q * 2;
#pragma unroll
        for (int j = 0; j < X_ROUNDS; ++j) {
            const int h = hb + x_r[j];
            const bool live = ok && x_g[j] >= 0 && (unsigned)h < (unsigned)p.H;
            unsigned v = live ? (unsigned)(xb + h * p.W * 2 + x_g[j]) : 0x80000000u;
            // (the empty asm keeps ONE load with a selected offset; left to itself the compiler puts a load on
            // either side of a branch, and the second one waits for every load in flight)
            asm volatile("" : "+v"(v));
            xr[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, v, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < D_ROUNDS; ++j) {
            unsigned v = (ok && d_g[j] >= 0) ? (unsigned)(db + d_g[j]) : 0x80000000u;
            asm volatile("" : "+v"(v));
            dr[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, v, 0, 0);
        }
    };
    auto store_iter = [&](int buf, const u32x4 (&xr)[X_ROUNDS], const u32x4 (&dr)[D_ROUNDS]) {
        unsigned char* base = smem + buf * p.buf_bytes;
#pragma unroll
        for (int j = 0; j < X_ROUNDS; ++j) {
            if (SW == 2) {
                // eight pixels -> four of the even plane (low halves), four of the odd plane
                const u32x2 ev = {__builtin_amdgcn_perm(xr[j][1], xr[j][0], 0x05040100u),
                                  __builtin_amdgcn_perm(xr[j][3], xr[j][2], 0x05040100u)};
                const u32x2 od = {__builtin_amdgcn_perm(xr[j][1], xr[j][0], 0x07060302u),
                                  __builtin_amdgcn_perm(xr[j][3], xr[j][2], 0x07060302u)};
                *reinterpret_cast<u32x2*>(base + x_l[j]) = ev;
                *reinterpret_cast<u32x2*>(base + x_l[j] + (x_g[j] >= 0 ? plane_bytes : 8)) = od;
            } else {
                *reinterpret_cast<u32x4*>(base + x_l[j]) = xr[j];
            }
        }
#pragma unroll
        for (int j = 0; j < D_ROUNDS; ++j) *reinterpret_cast<u32x4*>(base + d_l[j]) = dr[j];
    };

    floatx16 acc[S];
#pragma unroll
    for (int s = 0; s < S; ++s)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[s][e] = 0.0f;
    float dbacc = 0.0f;
    // bias sums: the wavefronts of step parity 1 (which have one MFMA step fewer per row when the step
    // count is odd) read every step of their rows
    const bool do_db = p.db_out != nullptr && parity == 1;

    // the MFMA steps of the output row staged in buffer `buf`: this wavefront's step parity
    auto multiply = [&](int buf) {
        const unsigned char* base = smem + buf * p.buf_bytes;
        for (int st = parity; st < p.steps; st += 2) {
            const u32x4 a = *reinterpret_cast<const u32x4*>(base + a_addr + st * 32);
#pragma unroll
            for (int f = 0; f < SW; ++f) {
                // element range the taps of this plane touch, relative to the aligned packet at q - 4 .. q + 11
                int lo = 99, hi = -99;
#pragma unroll
                for (int s = 0; s < S; ++s)
                    if (tap_plane(s, PW, SW) == f) {
                        lo = min(lo, tap_shift(s, PW, SW));
                        hi = max(hi, tap_shift(s, PW, SW));
                    }
                if (lo > hi) continue;                            // no tap reads this plane
                const unsigned char* pb = base + b_row + f * plane_bytes + st * 32;
                uint32_t w[8];                                    // dwords of elements q - 4 .. q + 11
                if (SW == 2) {
                    // (4-byte reads of the dwords on either side would all fall into the 16 banks the
                    // 16-byte row pitch allows: four lanes per bank)
                    const u32x4 d0 = *reinterpret_cast<const u32x4*>(pb - 8);
                    const u32x4 d1 = *reinterpret_cast<const u32x4*>(pb + 8);
                    w[0] = d0[0]; w[1] = d0[1]; w[2] = d0[2]; w[3] = d0[3];
                    w[4] = d1[0]; w[5] = d1[1]; w[6] = d1[2]; w[7] = d1[3];
                } else {
                    const u32x4 d = *reinterpret_cast<const u32x4*>(pb);
                    w[2] = d[0]; w[3] = d[1]; w[4] = d[2]; w[5] = d[3];
                    const int first = (4 + lo) >> 1, last = (4 + hi + 7) >> 1;
                    w[0] = first <= 0 ? *reinterpret_cast<const uint32_t*>(pb - 8) : 0u;
                    w[1] = first <= 1 ? *reinterpret_cast<const uint32_t*>(pb - 4) : 0u;
                    w[6] = last >= 6 ? *reinterpret_cast<const uint32_t*>(pb + 16) : 0u;
                    w[7] = last >= 7 ? *reinterpret_cast<const uint32_t*>(pb + 20) : 0u;
                }
#pragma unroll
                for (int s = 0; s < S; ++s) {
                    if (tap_plane(s, PW, SW) != f) continue;
                    const int e0 = 4 + tap_shift(s, PW, SW), i = e0 >> 1;
                    u32x4 bv;
                    if (e0 & 1)
                        bv = u32x4{__builtin_amdgcn_alignbit(w[i + 1], w[i], 16), __builtin_amdgcn_alignbit(w[i + 2], w[i + 1], 16),
                                   __builtin_amdgcn_alignbit(w[i + 3], w[i + 2], 16), __builtin_amdgcn_alignbit(w[i + 4], w[i + 3], 16)};
                    else
                        bv = u32x4{w[i], w[i + 1], w[i + 2], w[i + 3]};
                    acc[s] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, bv), acc[s], 0, 0, 0);
                }
            }
            if (do_db) dbacc += sum8(a);
        }
        if (do_db)      // ... so they take the other parity's steps of their own rows as well
            for (int st = 0; st < p.steps; st += 2) dbacc += sum8(*reinterpret_cast<const u32x4*>(base + a_addr + st * 32));
    };

    if (g0 < g1) {
        __syncthreads();                         // zeros in place
        load_iter(g0, xr0, dr0);
        load_iter(g0 + 1, xr1, dr1);             // past the range: all zeros, never multiplied
        store_iter(0, xr0, dr0);
        __syncthreads();
        // Iteration at row g, staged in buffer b: request row g + 2 into the register set that was stored
        // last, multiply, store the other set (row g + 1) into the other buffer. Nobody reads that
        // buffer: its readers passed the last barrier.
        int g = g0;
        while (true) {
            load_iter(g + 2, xr0, dr0);
            multiply(0);
            store_iter(1, xr1, dr1);
            __syncthreads();
            g += 1;
            if (g >= g1) break;
            load_iter(g + 2, xr1, dr1);
            multiply(1);
            store_iter(0, xr0, dr0);
            __syncthreads();
            g += 1;
            if (g >= g1) break;
        }
    }

    // ---- add the two step parities' tiles through LDS (fixed order), one tap at a time
    float* red = reinterpret_cast<float*>(smem);             // [wavefront][16][64]
    float* __restrict__ out = p.out + (size_t)worker * p.K * p.ncol;
#pragma unroll
    for (int s = 0; s < S; ++s) {
        __syncthreads();
#pragma unroll
        for (int e = 0; e < 16; ++e) red[(wave * 16 + e) * 64 + lane] = acc[s][e];
        __syncthreads();
#pragma unroll
        for (int h = 0; h < 2 * 1024 / NT; ++h) {
            const int idx = tid + h * NT;                       // (k tile, e, lane)
            const int t = idx >> 10, e = (idx >> 6) & 15, l = idx & 63;
            const float v = red[(t * 16 + e) * 64 + l] + red[((t + 2) * 16 + e) * 64 + l];
            const int k = k0 + t * 32 + (e >> 2) * 8 + (l >> 5) * 4 + (e & 3);
            const int row = l & 31;
            if (k < p.K && row < p.cr) out[(size_t)k * p.ncol + row * S + s] = v;
        }
    }
    if (p.db_out != nullptr) {   // lanes l and l + 32 hold the two 8-pixel halves of row l's steps
        const float tot = dbacc + __shfl_xor(dbacc, 32);
        const int k = k0 + kt * 32 + (lane & 31);
        if (parity == 1 && khalf == 0 && k < p.K) p.db_out[(size_t)worker * p.K + k] = tot;
    }
}

bool fill_params(const ConvGeom& g, TapsWgradParams* out) {
    TapsWgradParams p{};
    if (g.sw != 1 && g.sw != 2) return false;
    if (g.C * g.R > 32 || g.C * g.R < 1) return false;
    if ((g.W & 7) || (g.Q & 15) || (g.x_ns & 7) || (g.y_ns & 7) || g.K < 32) return false;
    const long long xb = ((long long)(g.N - 1) * g.x_ns + (long long)g.C * g.H * g.W) * 2;
    const long long dyb = ((long long)(g.N - 1) * g.y_ns + (long long)g.K * g.P * g.Q) * 2;
    if (xb >= 0x7fffffffLL || dyb >= 0x7fffffffLL) return false;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q;
    p.R = g.R; p.sh = g.sh; p.ph = g.ph;
    p.x_ns = g.x_ns; p.dy_ns = g.y_ns;
    p.x_bytes = (unsigned)xb; p.dy_bytes = (unsigned)dyb;
    p.cr = g.C * g.R;
    p.ncol = p.cr * g.S;
    p.steps = g.Q / 16;
    p.xchunks = g.W / 8; p.dychunks = g.Q / 8;
    // a plane row holds the W / sw columns of its parity and every window of the steps (elements
    // q - 4 .. q + 11 around each aligned packet)
    const int org = plane_org(g.sw);
    int elems = org + p.steps * 16 + 4;
    if (elems < org + (g.W + g.sw - 1) / g.sw) elems = org + (g.W + g.sw - 1) / g.sw;
    p.ppitch = odd16_pitch(elems * 2);
    p.dpitch = odd16_pitch(g.Q * 2);
    p.x_tasks = p.cr * p.xchunks;
    p.d_tasks = KT * p.dychunks;
    if (p.x_tasks > X_ROUNDS * NT || p.d_tasks > D_ROUNDS * NT) return false;
    p.d_bytes = KT * p.dpitch;
    p.spare_off = p.d_bytes + g.sw * p.cr * p.ppitch;
    p.buf_bytes = p.spare_off + NT * 16;
    if (2LL * p.buf_bytes > 80 * 1024 || 2LL * p.buf_bytes < (NT / 64) * 16 * 64 * 4) return false;
    p.k_groups = (g.K + KT - 1) / KT;
    if (p.k_groups > 64) return false;
    p.rows_total = g.N * g.P;
    int workers = 512 / p.k_groups;                              // two workgroups per CU
    int rpw = (p.rows_total + workers - 1) / workers;
    if (rpw < 8) rpw = 8;                                        // a shorter range is mostly set-up and the final sum
    p.rows_per_worker = rpw;
    p.workers = (p.rows_total + rpw - 1) / rpw;
    p.div_p = make_fastdiv(g.P);
    *out = p;
    return true;
}

template <int S, int PW, int SW>
hipError_t launch_taps(const TapsWgradParams& p, hipStream_t st) {
    static_assert(tap_shift(0, PW, SW) >= -4 && tap_shift(S - 1, PW, SW) <= 4, "windows stay within q - 4 .. q + 11");
    const size_t lds = 2 * (size_t)p.buf_bytes;
    auto kern = wgrad_taps_bf16_kernel<S, PW, SW>;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    ProbeScope probe(st);
    (void)hipGetLastError();
    hipLaunchKernelGGL(kern, dim3((unsigned)(p.workers * p.k_groups)), dim3(NT), lds, st, p);
    return hipGetLastError();
}

// the filter shapes (columns, left padding, column stride) the kernel is built for
#define TAPS_SHAPES(X) X(7, 3, 2) X(7, 3, 1) X(5, 2, 2) X(5, 2, 1) X(3, 1, 2) X(3, 1, 1) X(1, 0, 2) X(1, 0, 1)

bool shape_known(int S, int pw, int sw) {
#define X(s, p, w) if (S == s && pw == p && sw == w) return true;
    TAPS_SHAPES(X)
#undef X
    return false;
}

}  // namespace

// On success *workers is the number of partial tiles the kernel writes.
bool wgrad_taps_bf16_applies(const ConvGeom& g, int* workers) {
    TapsWgradParams p;
    if (!shape_known(g.S, g.pw, g.sw) || !fill_params(g, &p)) return false;
    *workers = p.workers;
    return true;
}

hipError_t launch_wgrad_taps_bf16(const ConvGeom& g, const void* x, const void* dy, float* partials,
                                  float* db_partials, hipStream_t st) {
    TapsWgradParams p;
    if (!shape_known(g.S, g.pw, g.sw) || !fill_params(g, &p)) return hipErrorInvalidValue;
    p.x = (const uint16_t*)x; p.dy = (const uint16_t*)dy; p.out = partials; p.db_out = db_partials;
#define X(s, pd, w) if (g.S == s && g.pw == pd && g.sw == w) return launch_taps<s, pd, w>(p, st);
    TAPS_SHAPES(X)
#undef X
    return hipErrorInvalidValue;
}

}  // namespace purine

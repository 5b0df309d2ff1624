// bf16 weight gradient for layers with few filter elements per output channel, C*R*S <= 160, and a
// column stride of 1 or 2: the first layer of an image network (ConvBwdWeight of paper Figure 1(b)):
//
//     dw[k, c, r, s] = sum over (n, p, q) of dy[n, k, p, q] * x[n, c, sh*p - ph + r, sw*q - pw + s]
//
// As a GEMM this is [K] x [C*R*S] with the pixels as the reduction: a small output tile and a very
// long reduction that streams dy (the large operand) exactly once. The kernel is built around that:
//
//  * A workgroup of four wavefronts (one per SIMD, so that each may use the whole register file)
//    owns 64 output channels and ALL C*R*S columns; every wavefront holds the whole 64 x 160 tile in
//    accumulators (2 x 5 MFMA tiles of 32x32) and the wavefronts split the reduction: each takes
//    every fourth 16-pixel step. Nothing is shared between the wavefronts but the staged rows, and
//    their tiles are added through LDS once, at the very end.
//  * Workgroups are persistent over a contiguous range of (image, output row) pairs and walk it two
//    output rows at a time. Per iteration the dy rows of the 64 channels and the R input rows of
//    every channel that each output row touches are brought into LDS as 16-byte packets in the
//    order they lie in memory. The pass is bound by how many bytes a CU keeps in flight, so the
//    packets are requested TWO iterations ahead (two register sets, used in turn) and land in the
//    other half of a double buffer one iteration ahead (one barrier per iteration).
//  * With a column stride of 2 the eight consecutive pixels of an MFMA operand read every second
//    input column. The input rows are therefore de-interleaved on their way into LDS (a byte
//    permute per packet): one plane per column parity, so that column sw*q - pw + s is element
//    q + floor((s - pw) / sw) of plane (s - pw) mod sw and every operand is a window of 8
//    consecutive elements again. The window of a lane starts at its own column tap, i.e. at any
//    2-byte position: the lane reads the five aligned dwords around it and funnel-shifts.
//  * dy rows need no re-layout at all (8 consecutive pixels of one channel = one packet).
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

constexpr int NT = 256;             // four wavefronts, one per SIMD
constexpr int KT = 64;              // output channels per workgroup
constexpr int RI = 2;               // output rows per iteration (the load tables below tell the two apart by one bit)
constexpr int ORG = 8;              // element of a plane that holds index 0 (left halo before it)
constexpr int X_ROUNDS = 6;         // 16-byte packets per thread and iteration, at most: input rows
constexpr int D_ROUNDS = 8;         // ... and dy rows
constexpr int MAX_NCT = 5;          // column tiles of 32: C*R*S <= 160

// LDS pitch: at least `bytes`, an odd number of 16-byte packets, so that 16-byte reads of 8
// consecutive rows fall into distinct bank groups
inline int odd16_pitch(int bytes) {
    int packets = (bytes + 15) / 16;
    if ((packets & 1) == 0) packets += 1;
    return packets * 16;
}

struct ColsWgradParams {
    const uint16_t* x; const uint16_t* dy; float* out; float* db_out;
    int N, C, H, W, K, P, Q, R, S, sh, ph, pw;
    int x_ns, dy_ns;
    unsigned x_bytes, dy_bytes;
    int k_groups, workers;             // grid = workers * k_groups
    int rows_total, rows_per_worker;   // flattened (n, p) output rows; rows_per_worker is a multiple of RI
    int ncol;                          // C*R*S
    int ppitch, dpitch;                // LDS bytes per plane / per dy row
    int xchunks, dychunks;             // 16-byte packets per input row (W / 8) and dy row (Q / 8)
    int steps;                         // 16-pixel MFMA steps per output row: Q / 16
    int x_tasks, d_tasks;              // packets per iteration
    int d_bytes, buf_bytes;            // bytes of the dy rows of one buffer; of one whole buffer
    int spare_off;                     // offset of a buffer's spare packets (one per thread)
    FastDiv div_p;
};

__device__ __forceinline__ float sum8(const u32x4 u) {
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += __uint_as_float(u[i] << 16) + __uint_as_float(u[i] & 0xffff0000u);
    return s;
}

// NCT: column tiles of 32 (ceil(C*R*S / 32)); SW: column stride (1 or 2) = planes per input row
template <int NCT, int SW>
__global__ __launch_bounds__(NT, 1) void wgrad_cols_bf16_kernel(const ColsWgradParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    // buffer b at smem + b * buf_bytes: dy rows [RI][KT] of dpitch bytes, then planes [RI][R][C][SW] of ppitch bytes

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int khalf = lane >> 5;
    const int kg = blockIdx.x % p.k_groups, worker = blockIdx.x / p.k_groups;
    const int k0 = kg * KT;
    const int g0 = worker * p.rows_per_worker;
    const int g1 = min(g0 + p.rows_per_worker, p.rows_total);
    const int slot_bytes = p.R * p.C * SW * p.ppitch;          // planes of one output row

    // ---- once: zeros everywhere (halos of the planes, the channels past K)
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < 2 * p.buf_bytes / 16; i += NT) *reinterpret_cast<u32x4*>(smem + i * 16) = z;
    }

    // ---- this lane's operand windows: column (c, r, s) -> plane, first element, funnel shift
    int b_addr[NCT], b_sh[NCT];
    const int RS = p.R * p.S;
#pragma unroll
    for (int ct = 0; ct < NCT; ++ct) {
        const int col = min(ct * 32 + (lane & 31), p.ncol - 1);     // padding columns repeat the last one, never stored
        const int c = col / RS, rs = col - c * RS;
        const int r = rs / p.S, s = rs - r * p.S;
        const int t = s - p.pw;
        const int f = SW == 2 ? (t & 1) : 0;
        const int d = SW == 2 ? (t >> 1) : t;                        // floor((s - pw) / sw)
        const int byte = p.d_bytes + ((r * p.C + c) * SW + f) * p.ppitch + (ORG + d + khalf * 8) * 2;
        b_addr[ct] = byte & ~3;
        b_sh[ct] = (byte & 2) * 8;
    }
    const int a_addr = (lane & 31) * p.dpitch + khalf * 16;

    // ---- load tasks of this thread (fixed over the iterations)
    int x_g[X_ROUNDS], x_l[X_ROUNDS], x_r[X_ROUNDS], x_i[X_ROUNDS];
#pragma unroll
    for (int j = 0; j < X_ROUNDS; ++j) {
        const int t = tid + j * NT;
        const int chunk = t % p.xchunks, u = t / p.xchunks;
        const int c = u % p.C, v = u / p.C;
        const int r = v % p.R, i = v / p.R;
        const bool live = t < p.x_tasks;
        x_g[j] = live ? (c * p.H * p.W + chunk * 8) * 2 : -1;
        // a thread without a task in this round loads zeros (range check) and stores them into a spare
        // packet of its own behind the buffers: the loop below has no branch around loads or stores, which
        // lets the compiler wait for exactly the older register set
        x_l[j] = live ? p.d_bytes + ((i * p.R + r) * p.C + c) * SW * p.ppitch + (ORG + chunk * (8 / SW)) * 2
                      : p.spare_off + tid * 16;
        x_r[j] = r;
        x_i[j] = i;
    }
    int d_g[D_ROUNDS], d_l[D_ROUNDS], d_i[D_ROUNDS];
#pragma unroll
    for (int j = 0; j < D_ROUNDS; ++j) {
        const int t = tid + j * NT;
        const int chunk = t % p.dychunks, u = t / p.dychunks;
        const int k = u % KT, i = u / KT;
        const bool live = t < p.d_tasks;
        d_g[j] = (live && k0 + k < p.K) ? ((k0 + k) * p.P * p.Q + chunk * 8) * 2 : -1;
        d_l[j] = live ? (i * KT + k) * p.dpitch + chunk * 16 : p.spare_off + tid * 16;
        d_i[j] = i;
    }
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), (short)0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_dy =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.dy), (short)0, (int)p.dy_bytes, 0x00020000);
    u32x4 xr0[X_ROUNDS], dr0[D_ROUNDS], xr1[X_ROUNDS], dr1[D_ROUNDS];   // the two register sets

    // packets of the RI output rows starting at flattened row g (rows at or past g1, input rows outside
    // the image and channels past K come back as zeros: range-checked loads)
    auto load_iter = [&](int g, u32x4 (&xr)[X_ROUNDS], u32x4 (&dr)[D_ROUNDS]) {
        int xb[RI], db[RI], hb[RI];
        bool ok[RI];
#pragma unroll
        for (int i = 0; i < RI; ++i) {
            const int gi = g + i;
            ok[i] = gi < g1;
            const int n = fastdiv(gi, p.div_p), pp = gi - n * p.P;
            hb[i] = p.sh * pp - p.ph;
            xb[i] = n * p.x_ns * 2;
            db[i] = n * p.dy_ns * 2 + pp * p.Q * 2;
        }
#pragma unroll
        for (int j = 0; j < X_ROUNDS; ++j) {
            const bool second = x_i[j] != 0;
            const int h = (second ? hb[1] : hb[0]) + x_r[j];
            const bool live = (second ? ok[1] : ok[0]) && x_g[j] >= 0 && (unsigned)h < (unsigned)p.H;
            unsigned v = live ? (unsigned)((second ? xb[1] : xb[0]) + h * p.W * 2 + x_g[j]) : 0x80000000u;
            // (the empty asm keeps ONE load with a selected offset; left to itself the compiler puts a load on
            // either side of a branch, and the second one waits for every load in flight)
            asm volatile("" : "+v"(v));
            xr[j] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, v, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < D_ROUNDS; ++j) {
            const bool second = d_i[j] != 0;
            const bool live = (second ? ok[1] : ok[0]) && d_g[j] >= 0;
            unsigned v = live ? (unsigned)((second ? db[1] : db[0]) + d_g[j]) : 0x80000000u;
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
                *reinterpret_cast<u32x2*>(base + x_l[j] + (x_g[j] >= 0 ? p.ppitch : 8)) = od;
            } else {
                *reinterpret_cast<u32x4*>(base + x_l[j]) = xr[j];
            }
        }
#pragma unroll
        for (int j = 0; j < D_ROUNDS; ++j) {
            *reinterpret_cast<u32x4*>(base + d_l[j]) = dr[j];
        }
    };

    floatx16 acc[2][NCT];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < NCT; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;
    float dbacc[2] = {0.0f, 0.0f};
    const bool do_db = p.db_out != nullptr;

    // The MFMA steps of the output rows g, g + 1 staged in buffer `buf`. With one wavefront per SIMD nobody
    // else covers the LDS latency, so the operands of this wavefront's next step are read while the
    // MFMAs of the current one run.
    struct StepOperands { u32x4 a0, a1; uint32_t d[NCT][5]; };
    const int wave_s = __builtin_amdgcn_readfirstlane(wave);
    auto fetch = [&](const unsigned char* base, int t, StepOperands& o) {
        const int i = t >= p.steps ? 1 : 0;
        const int st = t - i * p.steps;
        const unsigned char* ap = base + i * KT * p.dpitch + a_addr + st * 32;
        o.a0 = *reinterpret_cast<const u32x4*>(ap);
        o.a1 = *reinterpret_cast<const u32x4*>(ap + 32 * p.dpitch);
        const unsigned char* bp = base + i * slot_bytes + st * 32;
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            const uint32_t* w = reinterpret_cast<const uint32_t*>(bp + b_addr[ct]);
#pragma unroll
            for (int e = 0; e < 5; ++e) o.d[ct][e] = w[e];
        }
    };
    auto multiply = [&](int g, int buf) {
        const unsigned char* base = smem + buf * p.buf_bytes;
        const int t_end = (g + 1 < g1 ? RI : 1) * p.steps;     // the second row of the last pair may not exist
        int t = wave_s;
        if (t >= t_end) return;
        StepOperands cur, nxt;
        fetch(base, t, cur);
        while (true) {
            const int tn = t + NT / 64;
            const bool more = tn < t_end;
            fetch(base, more ? tn : t, nxt);                    // past the end: the same step again, unused
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int ct = 0; ct < NCT; ++ct) {
                const uint32_t sh = (uint32_t)b_sh[ct];
                const u32x4 bv = {__builtin_amdgcn_alignbit(cur.d[ct][1], cur.d[ct][0], sh),
                                  __builtin_amdgcn_alignbit(cur.d[ct][2], cur.d[ct][1], sh),
                                  __builtin_amdgcn_alignbit(cur.d[ct][3], cur.d[ct][2], sh),
                                  __builtin_amdgcn_alignbit(cur.d[ct][4], cur.d[ct][3], sh)};
                acc[0][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, cur.a0), __builtin_bit_cast(bf16x8, bv), acc[0][ct], 0, 0, 0);
                acc[1][ct] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    __builtin_bit_cast(bf16x8, cur.a1), __builtin_bit_cast(bf16x8, bv), acc[1][ct], 0, 0, 0);
            }
            if (do_db) { dbacc[0] += sum8(cur.a0); dbacc[1] += sum8(cur.a1); }
            __builtin_amdgcn_sched_barrier(0);
            if (!more) break;
            cur = nxt;
            t = tn;
        }
    };

    if (g0 < g1) {
        __syncthreads();                         // zeros in place
        load_iter(g0, xr0, dr0);
        load_iter(g0 + RI, xr1, dr1);            // past the range: all zeros, never multiplied
        store_iter(0, xr0, dr0);
        __syncthreads();
        // Iteration at g with its rows in buffer b: request the rows of g + 2*RI into the register set
        // that was stored last, multiply, store the other set (rows of g + RI) into the other buffer.
        // Nobody reads that buffer: its readers passed the last barrier.
        int g = g0;
        while (true) {
            load_iter(g + 2 * RI, xr0, dr0);
            multiply(g, 0);
            store_iter(1, xr1, dr1);
            __syncthreads();
            g += RI;
            if (g >= g1) break;
            load_iter(g + 2 * RI, xr1, dr1);
            multiply(g, 1);
            store_iter(0, xr0, dr0);
            __syncthreads();
            g += RI;
            if (g >= g1) break;
        }
    }

    // ---- add the wavefronts' tiles through LDS (fixed order), one 32x32 tile at a time
    float* red = reinterpret_cast<float*>(smem);             // [wavefront][16][64]
    float* __restrict__ out = p.out + (size_t)worker * p.K * p.ncol;
#pragma unroll
    for (int kt = 0; kt < 2; ++kt) {
#pragma unroll
        for (int ct = 0; ct < NCT; ++ct) {
            __syncthreads();
#pragma unroll
            for (int e = 0; e < 16; ++e) red[(wave * 16 + e) * 64 + lane] = acc[kt][ct][e];
            __syncthreads();
#pragma unroll
            for (int h = 0; h < 1024 / NT; ++h) {
                const int idx = tid + h * NT;
                const int e = idx >> 6, l = idx & 63;
                float s = 0.0f;
#pragma unroll
                for (int w = 0; w < NT / 64; ++w) s += red[(w * 16 + e) * 64 + l];
                const int k = k0 + kt * 32 + (e >> 2) * 8 + (l >> 5) * 4 + (e & 3);
                const int col = ct * 32 + (l & 31);
                if (k < p.K && col < p.ncol) out[(size_t)k * p.ncol + col] = s;
            }
        }
    }
    if (do_db) {   // lanes l and l + 32 hold the two 8-pixel halves of row l's steps
        __syncthreads();
#pragma unroll
        for (int kt = 0; kt < 2; ++kt) {
            const float tot = dbacc[kt] + __shfl_xor(dbacc[kt], 32);
            if (khalf == 0) red[wave * KT + kt * 32 + lane] = tot;
        }
        __syncthreads();
        if (tid < KT && k0 + tid < p.K) {
            float s = 0.0f;
#pragma unroll
            for (int w = 0; w < NT / 64; ++w) s += red[w * KT + tid];
            p.db_out[(size_t)worker * p.K + k0 + tid] = s;
        }
    }
}

bool fill_params(const ConvGeom& g, ColsWgradParams* out) {
    ColsWgradParams p{};
    if (g.sw != 1 && g.sw != 2) return false;
    const int ncol = g.C * g.R * g.S;
    if (ncol > MAX_NCT * 32 || ncol < 1) return false;
    if ((g.W & 7) || (g.Q & 15) || (g.x_ns & 7) || (g.y_ns & 7) || g.K < 32) return false;
    const long long xb = ((long long)(g.N - 1) * g.x_ns + (long long)g.C * g.H * g.W) * 2;
    const long long dyb = ((long long)(g.N - 1) * g.y_ns + (long long)g.K * g.P * g.Q) * 2;
    if (xb >= 0x7fffffffLL || dyb >= 0x7fffffffLL) return false;
    // floor((s - pw) / sw) over the taps: the halo the planes need on either side
    const int d_min = g.sw == 2 ? ((0 - g.pw) >> 1) : -g.pw;
    const int d_max = g.sw == 2 ? ((g.S - 1 - g.pw) >> 1) : g.S - 1 - g.pw;
    if (ORG + d_min < 0) return false;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q;
    p.R = g.R; p.S = g.S; p.sh = g.sh; p.ph = g.ph; p.pw = g.pw;
    p.x_ns = g.x_ns; p.dy_ns = g.y_ns;
    p.x_bytes = (unsigned)xb; p.dy_bytes = (unsigned)dyb;
    p.ncol = ncol;
    p.steps = g.Q / 16;
    p.xchunks = g.W / 8; p.dychunks = g.Q / 8;
    // a plane holds the row's W / sw columns of its parity and every window of the steps (5 dwords from
    // the aligned start of the right-most tap)
    int elems = ORG + p.steps * 16 + (d_max > 0 ? d_max : 0) + 4;
    if (elems < ORG + (g.W + g.sw - 1) / g.sw) elems = ORG + (g.W + g.sw - 1) / g.sw;
    p.ppitch = odd16_pitch(elems * 2);
    p.dpitch = odd16_pitch(g.Q * 2);
    p.x_tasks = RI * g.R * g.C * p.xchunks;
    p.d_tasks = RI * KT * p.dychunks;
    if (p.x_tasks > X_ROUNDS * NT || p.d_tasks > D_ROUNDS * NT) return false;
    p.d_bytes = RI * KT * p.dpitch;
    p.spare_off = p.d_bytes + RI * g.R * g.C * g.sw * p.ppitch;
    p.buf_bytes = p.spare_off + NT * 16;
    if (2LL * p.buf_bytes > 150 * 1024 || 2LL * p.buf_bytes < (NT / 64) * 16 * 64 * 4) return false;
    p.k_groups = (g.K + KT - 1) / KT;
    if (p.k_groups > 32) return false;
    p.rows_total = g.N * g.P;
    int workers = 256 / p.k_groups;                              // one workgroup per CU (its wavefronts want all registers)
    int rpw = (p.rows_total + workers - 1) / workers;
    rpw = (rpw + RI - 1) / RI * RI;
    if (rpw < 4 * RI) rpw = 4 * RI;                              // a range shorter than that is mostly set-up and the final sum
    p.rows_per_worker = rpw;
    p.workers = (p.rows_total + rpw - 1) / rpw;
    p.div_p = make_fastdiv(g.P);
    *out = p;
    return true;
}

template <int NCT>
hipError_t launch_nct(const ColsWgradParams& p, int sw, hipStream_t st) {
    const size_t lds = 2 * (size_t)p.buf_bytes;
    auto kern = sw == 2 ? wgrad_cols_bf16_kernel<NCT, 2> : wgrad_cols_bf16_kernel<NCT, 1>;
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

}  // namespace

// On success *workers is the number of partial tiles the kernel writes.
bool wgrad_cols_bf16_applies(const ConvGeom& g, int* workers) {
    ColsWgradParams p;
    if (!fill_params(g, &p)) return false;
    *workers = p.workers;
    return true;
}

hipError_t launch_wgrad_cols_bf16(const ConvGeom& g, const void* x, const void* dy, float* partials,
                                  float* db_partials, hipStream_t st) {
    ColsWgradParams p;
    if (!fill_params(g, &p)) return hipErrorInvalidValue;
    p.x = (const uint16_t*)x; p.dy = (const uint16_t*)dy; p.out = partials; p.db_out = db_partials;
    switch ((p.ncol + 31) / 32) {
        case 1: return launch_nct<1>(p, g.sw, st);
        case 2: return launch_nct<2>(p, g.sw, st);
        case 3: return launch_nct<3>(p, g.sw, st);
        case 4: return launch_nct<4>(p, g.sw, st);
        default: return launch_nct<5>(p, g.sw, st);
    }
}

}  // namespace purine

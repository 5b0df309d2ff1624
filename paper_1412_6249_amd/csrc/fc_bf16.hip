// bf16 fully-connected layer (the fully-connected layers of section 3.3): the two gradient passes
// whose shape the convolution kernels serve badly.
//
// Weight gradient   dw[k][c] = sum_n dy[n][k] * x[n][c],   dy, x bf16, dw fp32,
// on the transposed matrices dyT [K x N] and xT [C x N], whose rows are the reduction axis.
// The reduction is only as long as the batch, so the pass is bound by writing dw (K*C*4 bytes; both
// operands together are a few MB and stay in L2): one workgroup owns a 128 x 128 tile of dw and
// runs the whole reduction for it, so there are no partial sums and no second pass. Each of the four
// wavefronts holds a 64 x 64 quarter in 2 x 2 accumulators of v_mfma_f32_32x32x16_bf16; dy gives
// the row operand and x the column operand, so a lane's 16 results of one accumulator sit in one
// column c of 16 rows k, and the 32 lanes of a half wavefront store 128 consecutive bytes of a row
// of dw. The operand rows of a 64-sample chunk of the batch go through LDS (row pitch 144 bytes:
// the 16-byte reads of 16 lanes in consecutive rows fall into different banks); the next chunk is
// fetched into registers while the current one is multiplied.
//
// Data gradient   dx[n][c] = sum_k dy[n][k] * w[k][c],   all bf16,
// is bound by reading w once (K*C*2 bytes). The MFMA wants 8 consecutive reduction elements per lane,
// and w has the reduction axis k outermost, so a workgroup stages chunks of 32 rows of w (128
// columns, 16-byte packets straight from the rows) in LDS as they are and each lane collects the 8
// values of its column with 2-byte LDS reads; dy rows have k innermost and are staged and read in
// 16-byte packets. A workgroup owns 128 rows n x 128 columns c of one slice of the reduction
// (blockIdx.y); with more than one slice the fp32 tiles go to scratch and a second kernel adds the
// slices in slice order and rounds once (fixed order, no atomics).
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "common.h"

namespace purine {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int TK = 128, TC = 128;       // tile of dw: rows k, columns c
constexpr int NCH = 64;                 // samples per staged chunk
constexpr int PITCH = NCH * 2 + 16;     // bytes per staged row
constexpr int PK_ROW = NCH / 8;         // 16-byte packets per staged row
constexpr int PK_T = TK * PK_ROW / 256; // packets per thread and operand

__global__ __launch_bounds__(256) void fc_wgrad_bf16_kernel(const uint16_t* __restrict__ dyT,
                                                            const uint16_t* __restrict__ xT, float* dw, int N, int K,
                                                            int C, int tiles_c, int accumulate) {
    __shared__ uint4 lds[(TK + TC) * PITCH / 16];
    char* const As = reinterpret_cast<char*>(lds);
    char* const Bs = As + TK * PITCH;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wy = wave >> 1, wx = wave & 1, i = lane & 31, h = lane >> 5;
    const int k0 = (int)(blockIdx.x / tiles_c) * TK, c0 = (int)(blockIdx.x % tiles_c) * TC;

    uint4 ra[PK_T], rb[PK_T];
    // N is a multiple of 8: a packet lies wholly inside a row or wholly behind its end
    auto fetch = [&](int n0) {
#pragma unroll
        for (int j = 0; j < PK_T; ++j) {
            const int p = tid + 256 * j, row = p / PK_ROW, n = n0 + (p % PK_ROW) * 8;
            ra[j] = make_uint4(0, 0, 0, 0);
            rb[j] = make_uint4(0, 0, 0, 0);
            if (n < N) {
                if (k0 + row < K) ra[j] = *reinterpret_cast<const uint4*>(dyT + (size_t)(k0 + row) * N + n);
                if (c0 + row < C) rb[j] = *reinterpret_cast<const uint4*>(xT + (size_t)(c0 + row) * N + n);
            }
        }
    };
    auto stage = [&]() {
#pragma unroll
        for (int j = 0; j < PK_T; ++j) {
            const int p = tid + 256 * j, off = (p / PK_ROW) * PITCH + (p % PK_ROW) * 16;
            *reinterpret_cast<uint4*>(As + off) = ra[j];
            *reinterpret_cast<uint4*>(Bs + off) = rb[j];
        }
    };

    floatx16 acc[2][2];
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[a][b][v] = 0.0f;

    const char* const arow = As + (wy * 64 + i) * PITCH + h * 16;
    const char* const brow = Bs + (wx * 64 + i) * PITCH + h * 16;
    fetch(0);
    for (int n0 = 0; n0 < N; n0 += NCH) {
        if (n0) __syncthreads();   // the previous chunk has been read by every wavefront
        stage();
        __syncthreads();
        if (n0 + NCH < N) fetch(n0 + NCH);
        const int left = N - n0;
        const int steps = left >= NCH ? NCH / 16 : (left + 15) / 16;   // a half step at the end reads staged zeros
        for (int s = 0; s < steps; ++s) {
            const bf16x8 a0 = *reinterpret_cast<const bf16x8*>(arow + s * 32);
            const bf16x8 a1 = *reinterpret_cast<const bf16x8*>(arow + 32 * PITCH + s * 32);
            const bf16x8 b0 = *reinterpret_cast<const bf16x8*>(brow + s * 32);
            const bf16x8 b1 = *reinterpret_cast<const bf16x8*>(brow + 32 * PITCH + s * 32);
            acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b0, acc[0][0], 0, 0, 0);
            acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a0, b1, acc[0][1], 0, 0, 0);
            acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b0, acc[1][0], 0, 0, 0);
            acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a1, b1, acc[1][1], 0, 0, 0);
        }
    }

    // accumulator element v of lane (i, h): row 8*(v/4) + 4*h + v%4, column i of its 32 x 32 tile
#pragma unroll
    for (int a = 0; a < 2; ++a)
#pragma unroll
        for (int b = 0; b < 2; ++b) {
            const int col = c0 + wx * 64 + b * 32 + i;
            if (col >= C) continue;
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = k0 + wy * 64 + a * 32 + 8 * (v / 4) + 4 * h + (v % 4);
                if (row >= K) continue;
                float* const o = dw + (size_t)row * C + col;
                __builtin_nontemporal_store(accumulate ? *o + acc[a][b][v] : acc[a][b][v], o);
            }
        }
}

// ---- data gradient -------------------------------------------------------------------------------
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

constexpr int DN = 128;                           // rows n of a tile of dx
constexpr int DK_UNIT = 64;                       // slices of the reduction are multiples of this
constexpr int D_COLS = 128;                       // columns c of a tile of dx

__device__ __forceinline__ uint32_t pack2(float lo, float hi) {   // round to nearest even
    const floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}

// DC: columns c of a tile (128 or 64: a wavefront takes 32 columns and all 128 or 64 of the rows).
// DKC: reduction elements per staged chunk (32: two LDS buffers and one barrier per chunk; 64: one
// buffer and two barriers).
// grid: x = column tiles x row tiles, y = slices of the reduction (k_per_slice is a multiple of DKC).
// One slice: bf16 results straight to dx; more: fp32 tiles to partial[slice][N][C].
template <int DC, int DKC>
__global__ __launch_bounds__(256) void fc_dgrad_bf16_kernel(const uint16_t* __restrict__ dy, const uint16_t* __restrict__ w,
                                                            uint16_t* __restrict__ dx, float* __restrict__ partial, int N,
                                                            int K, int C, int tiles_c, int k_per_slice) {
    constexpr int DB_PITCH = DC * 2 + 16;             // staged row of w (c innermost)
    constexpr int DA_PITCH = DKC * 2 + 16;            // staged row of dy (k innermost)
    constexpr int D_STAGE = DKC * DB_PITCH + DN * DA_PITCH;
    constexpr int NBUF = 2 * D_STAGE <= 64 * 1024 ? 2 : 1;
    constexpr int CW = DC / 32, RW = 4 / CW, NA = 4 / RW;   // wavefronts along c and n, accumulators each
    constexpr int WPK = DKC * DC / 8 / 256;           // packets of w per thread and chunk
    constexpr int APK = DN * DKC / 8 / 256;           // packets of dy per thread and chunk
    __shared__ uint4 lds[NBUF * D_STAGE / 16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, i = lane & 31, h = lane >> 5;
    const int wc = wave % CW, wr = wave / CW;
    const int c0 = (int)(blockIdx.x % tiles_c) * DC, n0 = (int)(blockIdx.x / tiles_c) * DN;
    const int kb = (int)blockIdx.y * k_per_slice;
    const int ke = kb + k_per_slice < K ? kb + k_per_slice : K;

    uint4 rw[WPK], ra[APK];
    // K and C are multiples of 8 and a slice starts at a multiple of DKC: packets are whole or absent
    auto fetch = [&](int k0) {
#pragma unroll
        for (int j = 0; j < WPK; ++j) {
            const int p = tid + 256 * j;
            const int kw = k0 + p / (DC / 8), c = c0 + (p % (DC / 8)) * 8;
            rw[j] = make_uint4(0, 0, 0, 0);
            if (kw < ke && c < C) rw[j] = *reinterpret_cast<const uint4*>(w + (size_t)kw * C + c);
        }
#pragma unroll
        for (int j = 0; j < APK; ++j) {
            const int p = tid + 256 * j;
            const int n = n0 + p / (DKC / 8), ka = k0 + (p % (DKC / 8)) * 8;
            ra[j] = make_uint4(0, 0, 0, 0);
            if (n < N && ka < ke) ra[j] = *reinterpret_cast<const uint4*>(dy + (size_t)n * K + ka);
        }
    };
    auto stage = [&](char* bs) {
        char* const as = bs + DKC * DB_PITCH;
#pragma unroll
        for (int j = 0; j < WPK; ++j) {
            const int p = tid + 256 * j;
            *reinterpret_cast<uint4*>(bs + (p / (DC / 8)) * DB_PITCH + (p % (DC / 8)) * 16) = rw[j];
        }
#pragma unroll
        for (int j = 0; j < APK; ++j) {
            const int p = tid + 256 * j;
            *reinterpret_cast<uint4*>(as + (p / (DKC / 8)) * DA_PITCH + (p % (DKC / 8)) * 16) = ra[j];
        }
    };

    floatx16 acc[NA];
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[a][v] = 0.0f;

    fetch(kb);
    int buf = 0;
    for (int k0 = kb; k0 < ke; k0 += DKC, buf ^= (NBUF - 1)) {
        // two buffers: the other one may still be read by slower wavefronts, this one was last read
        // two chunks ago, before the previous chunk's barrier. One buffer: wait for its readers.
        if (NBUF == 1 && k0 != kb) __syncthreads();
        char* const bs = reinterpret_cast<char*>(lds) + buf * D_STAGE;
        stage(bs);
        __syncthreads();
        if (k0 + DKC < ke) fetch(k0 + DKC);
        const char* const bcol = bs + (8 * h) * DB_PITCH + (wc * 32 + i) * 2;
        const char* const arow = bs + DKC * DB_PITCH + (wr * NA * 32 + i) * DA_PITCH + h * 16;
#pragma unroll
        for (int s = 0; s < DKC / 16; ++s) {
            uint32_t q[4];
#pragma unroll
            for (int t = 0; t < 4; ++t) {
                const uint32_t lo = *reinterpret_cast<const uint16_t*>(bcol + (s * 16 + 2 * t) * DB_PITCH);
                const uint32_t hi = *reinterpret_cast<const uint16_t*>(bcol + (s * 16 + 2 * t + 1) * DB_PITCH);
                q[t] = lo | (hi << 16);
            }
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 qv = {q[0], q[1], q[2], q[3]};
            const bf16x8 b = __builtin_bit_cast(bf16x8, qv);
#pragma unroll
            for (int a = 0; a < NA; ++a) {
                const bf16x8 av = *reinterpret_cast<const bf16x8*>(arow + a * 32 * DA_PITCH + s * 32);
                acc[a] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av, b, acc[a], 0, 0, 0);
            }
        }
    }

    // accumulator element v of lane (i, h): row 8*(v/4) + 4*h + v%4, column i of its 32 x 32 tile
    const int col = c0 + wc * 32 + i;
    if (col >= C) return;
#pragma unroll
    for (int a = 0; a < NA; ++a)
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int n = n0 + (wr * NA + a) * 32 + 8 * (v / 4) + 4 * h + (v % 4);
            if (n >= N) continue;
            if (gridDim.y > 1)
                partial[((size_t)blockIdx.y * N + n) * C + col] = acc[a][v];
            else
                dx[(size_t)n * C + col] = (uint16_t)pack2(acc[a][v], 0.0f);
        }
}

// dx = bf16(sum over the slices, in slice order), 8 elements per thread (N*C is a multiple of 8)
__global__ __launch_bounds__(256) void fc_dgrad_finish_kernel(const float* __restrict__ partial, uint16_t* __restrict__ dx,
                                                              size_t packets, size_t slice_elems, int slices) {
    const size_t stride = (size_t)gridDim.x * 256;
    for (size_t p = (size_t)blockIdx.x * 256 + threadIdx.x; p < packets; p += stride) {
        const float4* src = reinterpret_cast<const float4*>(partial + p * 8);
        float4 lo = src[0], hi = src[1];
        for (int s = 1; s < slices; ++s) {
            const float4* q = reinterpret_cast<const float4*>(partial + (size_t)s * slice_elems + p * 8);
            const float4 l2 = q[0], h2 = q[1];
            lo.x += l2.x; lo.y += l2.y; lo.z += l2.z; lo.w += l2.w;
            hi.x += h2.x; hi.y += h2.y; hi.z += h2.z; hi.w += h2.w;
        }
        reinterpret_cast<uint4*>(dx)[p] = make_uint4(pack2(lo.x, lo.y), pack2(lo.z, lo.w), pack2(hi.x, hi.y), pack2(hi.z, hi.w));
    }
}

}  // namespace

// Batches of whole 16-byte packets (a multiple of 8 samples); the tile count must fit the grid.
bool fc_wgrad_bf16_applies(int64_t N, int64_t C, int64_t K) {
    if (N < 8 || (N & 7) || C < 1 || K < 1) return false;
    const int64_t tiles = ((K + TK - 1) / TK) * ((C + TC - 1) / TC);
    return tiles <= 0x7fffffffLL && N <= 0x7fffffffLL && C <= 0x7fffffffLL && K <= 0x7fffffffLL;
}

// dyT [K x N] and xT [C x N] dense bf16 at 16-byte-aligned addresses, dw [K x C] dense fp32.
hipError_t launch_fc_wgrad_bf16(const void* dyT, const void* xT, float* dw, int N, int K, int C, bool accumulate,
                                hipStream_t st) {
    if (!fc_wgrad_bf16_applies(N, C, K)) return hipErrorInvalidValue;
    const int tiles_c = (C + TC - 1) / TC, tiles_k = (K + TK - 1) / TK;
    ProbeScope probe(st);
    (void)hipGetLastError();
    hipLaunchKernelGGL(fc_wgrad_bf16_kernel, dim3((unsigned)(tiles_k * tiles_c)), dim3(256), 0, st,
                       (const uint16_t*)dyT, (const uint16_t*)xT, dw, N, K, C, tiles_c, accumulate ? 1 : 0);
    return hipGetLastError();
}

// Rows of whole 16-byte packets (K and C multiples of 8). *slices: how many slices of the reduction
// run side by side; *k_per_slice: their length, a multiple of the staged chunk. Returns the scratch bytes (0 for one slice), or SIZE_MAX when the kernel does not apply.
size_t fc_dgrad_bf16_plan(int64_t N, int64_t C, int64_t K, int* slices, int* k_per_slice) {
    if (N < 1 || C < 8 || K < 8 || (C & 7) || (K & 7)) return SIZE_MAX;
    if (N > 0x7fffffffLL || C > 0x7fffffffLL || K > 0x7fffffffLL) return SIZE_MAX;
    // measured, 128 x 9216 over 4096 (72 tiles of 128 columns): 4 / 6 / 8 / 11 slices take 0.039 / 0.035 /
    // 0.037 / 0.042 ms with the second pass: more slices shorten the workgroups' serial chains of
    // chunks, fewer keep the fp32 tiles (slices * N * C * 4 bytes, written and read again) small
    // (64-column tiles and 64-element chunks measured the same at the same workgroup count)
    const int tgt = 384, cols = D_COLS;
    const int64_t tiles = ((N + DN - 1) / DN) * ((C + cols - 1) / cols);
    if (tiles > 0x7fffffffLL) return SIZE_MAX;
    const int64_t chunks = (K + DK_UNIT - 1) / DK_UNIT;
    int64_t want = (tgt + tiles - 1) / tiles;
    if (want > chunks / 2) want = chunks / 2;            // at least 128 reduction elements per slice
    if (want > 64) want = 64;
    if (want < 1) want = 1;
    const int64_t per = (chunks + want - 1) / want;      // chunks per slice
    const int64_t n_slices = (chunks + per - 1) / per;
    if (slices) *slices = (int)n_slices;
    if (k_per_slice) *k_per_slice = (int)(per * DK_UNIT);
    return n_slices > 1 ? (size_t)n_slices * (size_t)N * (size_t)C * 4 : 0;
}

// dy [N x K], w [K x C], dx [N x C] dense bf16 at 16-byte-aligned addresses; ws: the scratch
// fc_dgrad_bf16_plan asks for (16-byte aligned).
hipError_t launch_fc_dgrad_bf16(const void* dy, const void* w, void* dx, int N, int K, int C, void* ws, hipStream_t st) {
    int slices = 0, k_per_slice = 0;
    const size_t need = fc_dgrad_bf16_plan(N, C, K, &slices, &k_per_slice);
    if (need == SIZE_MAX || (need && !ws)) return hipErrorInvalidValue;
    const int tiles_c = (C + D_COLS - 1) / D_COLS, tiles_n = (N + DN - 1) / DN;
    const dim3 grid((unsigned)(tiles_c * tiles_n), (unsigned)slices);
    (void)hipGetLastError();
    {
        ProbeScope probe(st);
        hipLaunchKernelGGL((fc_dgrad_bf16_kernel<D_COLS, 32>), grid, dim3(256), 0, st, (const uint16_t*)dy, (const uint16_t*)w,
                           (uint16_t*)dx, (float*)ws, N, K, C, tiles_c, k_per_slice);
    }
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || slices == 1) return e;
    const size_t elems = (size_t)N * C, packets = elems / 8;
    const size_t blocks = (packets + 255) / 256;
    hipLaunchKernelGGL(fc_dgrad_finish_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(256), 0, st,
                       (const float*)ws, (uint16_t*)dx, packets, elems, slices);
    return hipGetLastError();
}

}  // namespace purine

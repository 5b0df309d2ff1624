// 1x1, unit-stride, unpadded convolution (the "cccp" / reduce / projection layers of NIN- and
// inception-style networks) as a streaming GEMM: Conv and ConvBwdData of paper Figure 1(b) for the
// case where the gather is the identity.
//
//     out[n][i][pix] = sum_j A[i][j] * in[n][j][pix]        A = W (forward) or W^T (backward-data)
//
// NCHW keeps the pixels of one channel contiguous, which is exactly the register layout the fp32
// MFMA wants for its B operand (lane l holds reduction row l/32, column l%32). So the activations
// never pass through LDS: every lane streams its TN adjacent pixels of channel row 2*ks + l/32
// straight from global memory into B fragments with one vector load per reduction step, eight steps
// ahead of their use. Column c of pixel tile t is pixel TN*c + t of the strip, so a lane's TN tiles
// are adjacent pixels on the way in and on the way out (vector stores). Only the small filter goes
// through LDS (transposed on the fly from KCRS, no repacked copy), shared by the four wavefronts of
// a workgroup, each of which owns a strip of 32*TN pixels and all TM*32 output channels of the row
// tile. There is no barrier in the reduction loop unless the filter has more than 128 input channels.
#include "pix_common.h"

namespace purine {
namespace pix {
namespace {

constexpr int CK = 128;      // input channels of the filter held in LDS at a time
constexpr int DEPTH = 8;     // reduction steps (2 channels each) the activation loads run ahead

template <typename T, int TN> struct Vec;
template <> struct Vec<float, 1> {
    typedef float raw;
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[1]) { v[0] = r; }
    static __device__ __forceinline__ raw pack(const float (&v)[1]) { return v[0]; }
};
template <> struct Vec<uint16_t, 1> {
    typedef uint16_t raw;
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[1]) { v[0] = __uint_as_float((uint32_t)r << 16); }
    static __device__ __forceinline__ raw pack(const float (&v)[1]);
};
template <> struct Vec<float, 2> {
    typedef float2 raw;
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[2]) { v[0] = r.x; v[1] = r.y; }
    static __device__ __forceinline__ raw pack(const float (&v)[2]) { return make_float2(v[0], v[1]); }
};
template <> struct Vec<float, 4> {
    typedef float4 raw;
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[4]) {
        v[0] = r.x; v[1] = r.y; v[2] = r.z; v[3] = r.w;
    }
    static __device__ __forceinline__ raw pack(const float (&v)[4]) { return make_float4(v[0], v[1], v[2], v[3]); }
};
__device__ __forceinline__ uint32_t bf16_rne(float f) {
    uint32_t u = __float_as_uint(f);
    uint32_t r = u + 0x7FFFu + ((u >> 16) & 1u);
    if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) r = 0x7FC00000u;
    return r >> 16;
}
__device__ __forceinline__ uint16_t Vec<uint16_t, 1>::pack(const float (&v)[1]) { return (uint16_t)bf16_rne(v[0]); }
template <> struct Vec<uint16_t, 2> {
    typedef uint32_t raw;
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[2]) {
        v[0] = __uint_as_float(r << 16); v[1] = __uint_as_float(r & 0xffff0000u);
    }
    static __device__ __forceinline__ raw pack(const float (&v)[2]) { return bf16_rne(v[0]) | (bf16_rne(v[1]) << 16); }
};
template <> struct Vec<uint16_t, 4> {
    typedef uint2 raw;
    static __device__ __forceinline__ void unpack(const raw& r, float (&v)[4]) {
        v[0] = __uint_as_float(r.x << 16); v[1] = __uint_as_float(r.x & 0xffff0000u);
        v[2] = __uint_as_float(r.y << 16); v[3] = __uint_as_float(r.y & 0xffff0000u);
    }
    static __device__ __forceinline__ raw pack(const float (&v)[4]) {
        return make_uint2(bf16_rne(v[0]) | (bf16_rne(v[1]) << 16), bf16_rne(v[2]) | (bf16_rne(v[3]) << 16));
    }
};

// Filter part into LDS: As[k][m] = A[i0 + m][c0 + k] for k < ck (ck <= CKMAX), m < TM*32, zero beyond
// the last output channel. Threads walk the contiguous direction of W; loads go out in batches of
// FILL before any of them is stored, so a batch costs one memory latency, not FILL of them.
template <typename T, bool TRANS, int TM, int CKMAX>
__device__ __forceinline__ void fill_filter(float* __restrict__ As, const T* __restrict__ wt, int i0, int c0,
                                            int ck, int Ci, int Co, int tid) {
    constexpr int BM = TM * 32, LD = BM + 1, FILL = 8;
    static_assert((CKMAX & (CKMAX - 1)) == 0 && CKMAX >= 32 && CKMAX <= 256, "thread mapping");
    if (!TRANS) {
        // W[i][j], j contiguous: thread = (k, m mod MSTEP); m advances by MSTEP per iteration
        constexpr int MSTEP = 256 / CKMAX;
        static_assert(BM % (MSTEP * FILL) == 0, "whole batches");
        const int k = tid & (CKMAX - 1), mh = tid / CKMAX;
        const bool k_ok = k < ck;
        const T* wk = wt + c0 + (k_ok ? k : 0);
#pragma unroll 1
        for (int it0 = 0; it0 < BM / MSTEP; it0 += FILL) {
            float tmp[FILL];
#pragma unroll
            for (int j = 0; j < FILL; ++j) {
                const int i = i0 + MSTEP * (it0 + j) + mh;
                const bool ok = k_ok & (i < Co);
                tmp[j] = Elem<T>::load(wk, ok ? i * Ci : 0);
                tmp[j] = ok ? tmp[j] : 0.0f;
            }
            if (k_ok) {
#pragma unroll
                for (int j = 0; j < FILL; ++j) As[k * LD + MSTEP * (it0 + j) + mh] = tmp[j];
            }
        }
    } else {
        // W[j][i], i contiguous: thread = (m within a 32-row block, k mod 8)
        const int tm = tid & 31, tk = tid >> 5;
#pragma unroll 1
        for (int it = 0; it < TM * (CKMAX / 8 / FILL); ++it) {
            const int a = it / (CKMAX / 8 / FILL), kb = (it % (CKMAX / 8 / FILL)) * FILL;
            const int m = a * 32 + tm;
            const bool i_ok = i0 + m < Co;
            const T* wm = wt + (i_ok ? i0 + m : 0);
            float tmp[FILL];
#pragma unroll
            for (int j = 0; j < FILL; ++j) {
                const int k = (kb + j) * 8 + tk;
                const bool ok = i_ok & (k < ck);
                tmp[j] = Elem<T>::load(wm, ok ? (c0 + k) * Co : 0);
                tmp[j] = ok ? tmp[j] : 0.0f;
            }
#pragma unroll
            for (int j = 0; j < FILL; ++j) {
                const int k = (kb + j) * 8 + tk;
                if (k < ck) As[k * LD + m] = tmp[j];
            }
        }
    }
}

// Epilogue of one 32-row MFMA tile whose TN pixel tiles are a lane's TN adjacent pixels: optional
// bias, ReLU, ReLU-gradient mask, accumulate; vector stores. What 8 rows need from memory is
// requested before the first of their stores, so the loads overlap instead of forming
// load-wait-store round trips.
// FWD: forward pass (bias / ReLU, no mask, no accumulate); otherwise backward-data (the reverse).
template <typename T, bool FUSED, int TN, bool FWD>
__device__ __forceinline__ void store_rows(const PixParams& p, floatx16 (&acc)[TN], int row0, size_t obase,
                                           const float* bias_lds, int i_tile0) {
    typedef typename Vec<T, TN>::raw raw_t;
    const T* __restrict__ bias = FWD ? (const T*)p.bias : nullptr;
    const bool has_mask = FUSED && !FWD && p.mask != nullptr, has_beta = !FWD && p.beta != 0.0f;
    const bool relu = FWD && p.relu;
    // One per-lane pointer to (row0, this lane's pixels); the 16 rows of the tile are uniform
    // multiples of the plane size away. The pointers are made opaque so that the compiler does not
    // turn every row's address into a 64-bit induction variable of the loops around the epilogue.
    T* orow = (T*)p.out + obase + (size_t)row0 * p.HoWo;
    const T* mrow = (const T*)p.mask + (has_mask ? obase + (size_t)row0 * p.HoWo : 0);
    asm volatile("" : "+v"(orow));
    asm volatile("" : "+v"(mrow));
    // rows per batch: what a batch needs from memory (mask, old output) is requested before the
    // first of its stores; fewer rows per batch where a row is four pixels wide (registers)
    constexpr int G = TN >= 4 ? 4 : (FUSED ? 16 : 8);
#pragma unroll
    for (int part = 0; part < 16 / G; ++part) {
        const int e0 = part * G;
        raw_t mk[G], old[FUSED ? 1 : G];   // the fused kernels rarely accumulate: no staging there
        if (has_mask) {
#pragma unroll
            for (int e = 0; e < G; ++e) {
                const int d = ((e0 + e) >> 2) * 8 + ((e0 + e) & 3);
                // a row past the last channel reads channel 0 of the same image instead (row0 itself may
                // already lie past Co, so "offset 0 from mrow" would not be inside the tensor)
                mk[e] = *reinterpret_cast<const raw_t*>(mrow + (row0 + d < p.Co ? d : -row0) * p.HoWo);
            }
        }
        if (!FUSED && has_beta) {
#pragma unroll
            for (int e = 0; e < G; ++e) {
                const int d = ((e0 + e) >> 2) * 8 + ((e0 + e) & 3);
                old[e] = *reinterpret_cast<const raw_t*>(orow + (row0 + d < p.Co ? d : -row0) * p.HoWo);
            }
        }
        floatx4 bq = {0.0f, 0.0f, 0.0f, 0.0f};   // bias of four consecutive rows: one 16-byte LDS read per quad
#pragma unroll
        for (int e = 0; e < G; ++e) {
            const int d = ((e0 + e) >> 2) * 8 + ((e0 + e) & 3);
            const int i = row0 + d;
            // (row0 + d - i_tile0 is a multiple of 4 at the start of a quad; rows past Co hold zeros)
            if (FUSED && bias && ((e0 + e) & 3) == 0) bq = *reinterpret_cast<const floatx4*>(&bias_lds[i - i_tile0]);
            if (i >= p.Co) continue;
            float v[TN];
#pragma unroll
            for (int b = 0; b < TN; ++b) v[b] = acc[b][e0 + e];
            if (FUSED) {
                if (bias) {
#pragma unroll
                    for (int b = 0; b < TN; ++b) v[b] += bq[(e0 + e) & 3];
                }
                if (relu) {
#pragma unroll
                    for (int b = 0; b < TN; ++b) v[b] = v[b] > 0.0f ? v[b] : 0.0f;
                }
                if (has_mask) {
                    float m[TN];
                    Vec<T, TN>::unpack(mk[e], m);
#pragma unroll
                    for (int b = 0; b < TN; ++b) v[b] = m[b] > 0.0f ? v[b] : 0.0f;
                }
            }
            if (has_beta) {
                float o[TN];
                if (FUSED) old[0] = *reinterpret_cast<const raw_t*>(orow + d * p.HoWo);
                Vec<T, TN>::unpack(old[FUSED ? 0 : e], o);
#pragma unroll
                for (int b = 0; b < TN; ++b) v[b] += o[b];
            }
            *reinterpret_cast<raw_t*>(orow + d * p.HoWo) = Vec<T, TN>::pack(v);
        }
    }
}

// p.wt is the KCRS filter itself (R = S = 1, so [K][C]); TRANS: backward-data (A = W^T).
template <typename T, bool TRANS, bool FUSED, int TM, int TN>
__global__ __launch_bounds__(256, (TM * TN <= 6 ? 3 : 2)) void gemm1x1_kernel(const PixParams p) {
    constexpr int BM = TM * 32;
    constexpr int LD = BM + 1;             // odd pitch: the transposing fill is conflict-free
    constexpr int STRIP = 32 * TN;         // pixels per wavefront
    typedef typename Vec<T, TN>::raw raw_t;

    __shared__ float As[CK * LD];
    __shared__ __attribute__((aligned(16))) float bias_s[FUSED ? BM : 4];   // read in 16-byte quads

    const T* __restrict__ in = (const T*)p.in;
    const T* __restrict__ wt = (const T*)p.wt;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int col = lane & 31, khalf = lane >> 5;

    const int tile = xcd_tile(blockIdx.x, p.tiles_i * p.tiles_pix);
    const int i0 = (tile % p.tiles_i) * BM;
    const int m0 = ((tile / p.tiles_i) * 4 + wave) * STRIP + col * TN;   // this lane's first pixel
    const bool live = m0 < p.M;                                          // M % TN == 0: all or none
    int n = 0, pix = 0;
    if (live) {
        n = fastdiv(m0, p.div_howo);
        pix = m0 - n * p.HoWo;
    }
    // this workgroup's part of the reduction: all of it, or split blockIdx.y's channels
    const int c_begin = p.splits > 1 ? (int)blockIdx.y * p.split_ci : 0;
    const int c_end = p.splits > 1 ? min(c_begin + p.split_ci, p.Ci) : p.Ci;
    // reduction step ks reads channel rows c_begin + 2*ks + khalf; KS steps in all (multiples of 16 channels)
    const int KS = (c_end - c_begin) >> 1;
    const T* src = in + (size_t)n * p.in_ns + (size_t)(c_begin + khalf) * p.HoWo + pix;
    const size_t step = (size_t)2 * p.HoWo;

    // Two register sets of DEPTH reduction steps each: the loads of the next group are all issued
    // before the first MFMA of the current group, so they have a whole group's MFMA time to land.
    raw_t bcur[DEPTH], bnext[DEPTH];
    int ks_issue = 0;                      // next reduction step whose load has not been issued
    auto issue_group = [&](raw_t (&dst)[DEPTH]) {
#pragma unroll
        for (int u = 0; u < DEPTH; ++u) {  // past the end the last row pair is read again, unused
            dst[u] = *reinterpret_cast<const raw_t*>(src);
            ++ks_issue;
            src += ks_issue < KS ? step : 0;
        }
    };
    issue_group(bcur);
    if (FUSED) stage_bias<T, BM, 256>(bias_s, p, i0, tid);   // ordered by the barrier after the filter fill

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

    for (int c0 = c_begin; c0 < c_end; c0 += CK) {
        const int ck = c_end - c0 < CK ? c_end - c0 : CK;
        if (c0 > c_begin) __syncthreads(); // everyone is done with the previous part of the filter
        fill_filter<T, TRANS, TM, CK>(As, wt, i0, c0, ck, p.Ci, p.Co, tid);
        __syncthreads();

        const float* a_ptr = &As[khalf * LD + col];
        float areg[2][TM];
#pragma unroll
        for (int a = 0; a < TM; ++a) areg[0][a] = a_ptr[a * 32];
        const int steps = ck >> 1;         // multiple of DEPTH
        for (int s0 = 0; s0 < steps; s0 += DEPTH) {
            issue_group(bnext);
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) {
                const int s = s0 + u;
                // next step's filter fragments (the row after the part's last one is never used)
                const int s_next = s + 1 < steps ? s + 1 : s;
#pragma unroll
                for (int a = 0; a < TM; ++a) areg[(u + 1) & 1][a] = a_ptr[s_next * 2 * LD + a * 32];
                __builtin_amdgcn_sched_barrier(0);
                float bv[TN];
                Vec<T, TN>::unpack(bcur[u], bv);
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(areg[u & 1][a], bv[b], acc[a][b], 0, 0, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int u = 0; u < DEPTH; ++u) bcur[u] = bnext[u];
        }
    }

    if (!live) return;
    if (p.splits > 1) {
        // raw fp32 tile of this split, dense [N][Co][Ho*Wo]; the second kernel applies the epilogue
        PixParams q = p;
        q.out = p.partial + (size_t)blockIdx.y * p.N * p.Co * p.HoWo;
        q.out_ns = p.Co * p.HoWo;
        q.beta = 0.0f; q.bias = nullptr; q.mask = nullptr; q.relu = 0;
        const size_t pbase = (size_t)n * q.out_ns + pix;
#pragma unroll
        for (int a = 0; a < TM; ++a) store_rows<float, false, TN, true>(q, acc[a], i0 + a * 32 + khalf * 4, pbase, bias_s, i0);
        return;
    }
    const size_t obase = (size_t)n * p.out_ns + pix;
#pragma unroll
    for (int a = 0; a < TM; ++a) store_rows<T, FUSED, TN, !TRANS>(p, acc[a], i0 + a * 32 + khalf * 4, obase, bias_s, i0);
}

// Second pass of the split reduction: out = epilogue(sum over splits, in order, of partial[s]), V
// consecutive pixels per thread.
template <typename T, int V>
__global__ __launch_bounds__(256) void gemm1x1_reduce_kernel(const PixParams p, int fwd) {
    const long long groups = (long long)p.N * p.Co * (p.HoWo / V);
    const size_t split_stride = (size_t)p.N * p.Co * p.HoWo;
    const int per_row = p.HoWo / V;
    for (long long gidx = (long long)blockIdx.x * 256 + threadIdx.x; gidx < groups; gidx += (long long)gridDim.x * 256) {
        const long long row = gidx / per_row;                  // n * Co + i
        const int pg = (int)(gidx - row * per_row);
        const int n = (int)(row / p.Co), i = (int)(row - (long long)n * p.Co);
        const float* src = p.partial + (size_t)row * p.HoWo + (size_t)pg * V;
        float v[V];
#pragma unroll
        for (int e = 0; e < V; ++e) v[e] = 0.0f;
        for (int s = 0; s < p.splits; ++s) {
#pragma unroll
            for (int e = 0; e < V; ++e) v[e] += src[(size_t)s * split_stride + e];
        }
        const size_t o = (size_t)n * p.out_ns + (size_t)i * p.HoWo + (size_t)pg * V;
        if (fwd && p.bias) {
            const float b = Elem<T>::load((const T*)p.bias, i);
#pragma unroll
            for (int e = 0; e < V; ++e) v[e] += b;
        }
        if (fwd && p.relu) {
#pragma unroll
            for (int e = 0; e < V; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
        }
        if (!fwd && p.mask) {
#pragma unroll
            for (int e = 0; e < V; ++e) v[e] = Elem<T>::load((const T*)p.mask, (int)(o + e)) > 0.0f ? v[e] : 0.0f;
        }
        if (!fwd && p.beta != 0.0f) {
#pragma unroll
            for (int e = 0; e < V; ++e) v[e] += Elem<T>::load((const T*)p.out, (int)(o + e));
        }
#pragma unroll
        for (int e = 0; e < V; ++e) Elem<T>::store((T*)p.out, (int)(o + e), v[e]);
    }
}

template <typename T, bool TRANS, bool FUSED, int TM, int TN>
hipError_t launch_one(const PixParams& p, hipStream_t st) {
    const long long total = (long long)p.tiles_i * p.tiles_pix;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    const unsigned splits = p.splits > 1 ? (unsigned)p.splits : 1u;
    hipLaunchKernelGGL((gemm1x1_kernel<T, TRANS, FUSED, TM, TN>), dim3((unsigned)total, splits), dim3(256), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess || splits == 1) return e;
    const long long groups = (long long)p.N * p.Co * (p.HoWo / TN);
    const unsigned blocks = (unsigned)((groups + 255) / 256 > 8192 ? 8192 : (groups + 255) / 256);
    hipLaunchKernelGGL((gemm1x1_reduce_kernel<T, TN>), dim3(blocks), dim3(256), 0, st, p, TRANS ? 0 : 1);
    return hipGetLastError();
}

template <typename T, bool TRANS, bool FUSED>
hipError_t by_shape(const PixParams& p, int tm, int tn, hipStream_t st) {
    switch (tm * 10 + tn) {
        case 31: return launch_one<T, TRANS, FUSED, 3, 1>(p, st);
        case 21: return launch_one<T, TRANS, FUSED, 2, 1>(p, st);
        case 12: return launch_one<T, TRANS, FUSED, 1, 2>(p, st);
        case 22: return launch_one<T, TRANS, FUSED, 2, 2>(p, st);
        case 32: return launch_one<T, TRANS, FUSED, 3, 2>(p, st);
        case 14: return launch_one<T, TRANS, FUSED, 1, 4>(p, st);
        case 24: return launch_one<T, TRANS, FUSED, 2, 4>(p, st);
        default: return hipErrorInvalidValue;
    }
}

template <typename T>
hipError_t by_mode(const PixParams& p, bool trans, int tm, int tn, hipStream_t st) {
    const bool fused = p.bias || p.relu || p.mask;
    if (!trans) return fused ? by_shape<T, false, true>(p, tm, tn, st) : by_shape<T, false, false>(p, tm, tn, st);
    return fused ? by_shape<T, true, true>(p, tm, tn, st) : by_shape<T, true, false>(p, tm, tn, st);
}

}  // namespace

// tm, tn: MFMA tiles per wavefront (output channels / 32, pixels per lane). The caller has checked
// that the layer is 1x1 / stride 1 / no padding, Ci % 16 == 0, Ho*Wo % tn == 0 and that in, out
// and mask are aligned to tn elements.
hipError_t dispatch_gemm1x1(const PixParams& p, int dtype, bool trans, int tm, int tn, hipStream_t st) {
    if (p.Ci < 2 * DEPTH || (p.Ci & 15) || (p.HoWo % tn) != 0) return hipErrorInvalidValue;
    if (p.splits > 1 && (!p.partial || p.split_ci < CK || p.split_ci % CK != 0)) return hipErrorInvalidValue;
    return dtype == PURINE_F32 ? by_mode<float>(p, trans, tm, tn, st) : by_mode<uint16_t>(p, trans, tm, tn, st);
}

}  // namespace pix
}  // namespace purine

// Pixel-major implicit-GEMM convolution for gfx950: forward and backward-data.
//
// Both passes of the convolution operators (paper Figure 1(b)) are the contraction
//     out[n, i, ho, wo] = sum_{kk = (ci, r, s)} A[i, kk] * G[kk, (n, ho, wo)]
// where G is the patch matrix of the gathered tensor. G is never stored in HBM: each workgroup
// builds a BK x BN slab of it in LDS straight from the NCHW tensor (lanes run along pixels, so the
// loads are coalesced along W), multiplies it with a BK x BM slab of the filter matrix on the
// fp32 MFMA units, and keeps the BM x BN output tile in accumulator registers.
//   forward       : in = x,  i = k (output channel), kk = (c, r, s), hi = ho*sh - ph + r
//   backward-data : in = dy, i = c (input channel),  kk = (k, r, s), hi = (ho + ph - r)/sh if exact
// MFMA operand roles: A rows = channels, B columns = pixels, so each accumulator register holds 32
// consecutive pixels of one channel and the NCHW stores are 128-byte coalesced.
#include "common.h"

namespace purine {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;  // slab depth along the reduction

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p, int i) { return p[i]; }
    static __device__ __forceinline__ void store(float* p, int i, float v) { p[i] = v; }
};
template <> struct Elem<uint16_t> {  // bfloat16 bit patterns
    static __device__ __forceinline__ float load(const uint16_t* p, int i) {
        return __uint_as_float(((uint32_t)p[i]) << 16);
    }
    static __device__ __forceinline__ void store(uint16_t* p, int i, float v) {
        uint32_t u = __float_as_uint(v);
        uint32_t r = u + 0x7FFFu + ((u >> 16) & 1u);          // round to nearest even
        if ((u & 0x7F800000u) == 0x7F800000u && (u & 0x007FFFFFu)) r = 0x7FC00000u;  // NaN
        p[i] = (uint16_t)(r >> 16);
    }
};

// MODE 0 = forward, MODE 1 = backward-data. Workgroup = WM x WN wavefronts, each owning TM x TN
// MFMA tiles of 32 x 32.
template <typename T, int MODE, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void igemm_pix_kernel(const PixGemmParams p) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    constexpr int LDA = BM + 2;   // +2: the transposed filter-slab store hits distinct banks
    constexpr int LDB = BN;
    static_assert(NT % BN == 0 || BN % NT == 0, "pixel mapping");
    constexpr int B_COLS = BN > NT ? BN / NT : 1;      // pixel columns per thread
    constexpr int B_RPP = BN > NT ? 1 : NT / BN;       // slab rows covered per pass
    constexpr int B_PASSES = BK / B_RPP;
    static_assert(BK % B_RPP == 0, "row mapping");
    constexpr int A_RPP = NT / BK;                      // filter rows (channels) per pass
    constexpr int A_PASSES = (BM + A_RPP - 1) / A_RPP;

    __shared__ float As[2][BK * LDA];
    __shared__ float Bs[2][BK * LDB];

    const T* __restrict__ in = (const T*)p.in;
    const T* __restrict__ wt = (const T*)p.wt;
    T* __restrict__ out = (T*)p.out;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    // Consecutive workgroup ids land on different XCDs (8 per chip, each with its own L2). Give each
    // XCD a contiguous run of tiles so that neighbouring pixel tiles share halo rows in one L2.
    int tile = blockIdx.x;
    {
        const int total = p.tiles_i * p.tiles_pix;
        const int per = total >> 3;
        if (per > 0 && tile < per * 8) tile = (tile & 7) * per + (tile >> 3);
    }
    const int i0 = (tile % p.tiles_i) * BM;
    const int j0 = (tile / p.tiles_i) * BN;

    // ---- per-thread pixel bookkeeping for the gather (fixed for the whole kernel) ----
    int g_base[B_COLS], g_h[B_COLS], g_w[B_COLS];
    int g_hr[B_COLS], g_wr[B_COLS];   // backward-data with stride > 1: residues of (ho+ph), (wo+pw)
#pragma unroll
    for (int cidx = 0; cidx < B_COLS; ++cidx) {
        const int pix = j0 + (tid % BN) + cidx * NT;
        if (pix < p.M) {
            const int n = fastdiv(pix, p.div_howo);
            const int rem = pix - n * p.HoWo;
            const int ho = fastdiv(rem, p.div_wo);
            const int wo = rem - ho * p.Wo;
            if (MODE == 0) {
                g_h[cidx] = ho * p.sh - p.ph;
                g_w[cidx] = wo * p.sw - p.pw;
                g_hr[cidx] = g_wr[cidx] = 0;
            } else {
                const int th = ho + p.ph, tw = wo + p.pw;
                g_h[cidx] = fastdiv(th, p.div_sh);
                g_w[cidx] = fastdiv(tw, p.div_sw);
                g_hr[cidx] = th - g_h[cidx] * p.sh;
                g_wr[cidx] = tw - g_w[cidx] * p.sw;
            }
            g_base[cidx] = n * p.Ci * p.HiWi;
        } else {
            g_base[cidx] = -1;  // pixel beyond the tensor: contributes zeros
            g_h[cidx] = g_w[cidx] = g_hr[cidx] = g_wr[cidx] = 0;
        }
    }
    const int b_row = __builtin_amdgcn_readfirstlane(tid / BN);  // uniform per wavefront (BN >= 64)
    const int a_kk = tid % BK;
    const int a_i = tid / BK;

    float a_reg[A_PASSES];
    float b_reg[B_PASSES][B_COLS];

    auto load_slab = [&](int slab) {
        // filter slab: A[i, kk] for kk = slab*BK + a_kk
        {
            const int kk = slab * BK + a_kk;
            const bool kv = kk < p.Kg;
            const int ci = fastdiv(kv ? kk : 0, p.div_rs);
            const int rs = (kv ? kk : 0) - ci * p.RS;
            const int base = ci * p.a_ci_stride + rs;
#pragma unroll
            for (int ps = 0; ps < A_PASSES; ++ps) {
                const int il = a_i + ps * A_RPP;
                const int i = i0 + il;
                a_reg[ps] = (kv && il < BM && i < p.Co) ? Elem<T>::load(wt, base + i * p.a_i_stride) : 0.0f;
            }
        }
        // patch slab: G[kk, pixel]; kk is uniform across the wavefront, so (ci, r, s) is scalar work
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps) {
            const int kk = slab * BK + ps * B_RPP + b_row;
            const bool kv = kk < p.Kg;
            const int kq = kv ? kk : 0;
            const int ci = fastdiv(kq, p.div_rs);
            const int rs = kq - ci * p.RS;
            const int r = fastdiv(rs, p.div_s);
            const int s = rs - r * p.S;
            int rq = 0, rr = 0, sq = 0, sr = 0;
            if (MODE == 1) {
                rq = fastdiv(r, p.div_sh); rr = r - rq * p.sh;
                sq = fastdiv(s, p.div_sw); sr = s - sq * p.sw;
            }
            const int plane = ci * p.HiWi;
#pragma unroll
            for (int cidx = 0; cidx < B_COLS; ++cidx) {
                int hi, wi;
                bool ok = kv && g_base[cidx] >= 0;
                if (MODE == 0) {
                    hi = g_h[cidx] + r;
                    wi = g_w[cidx] + s;
                } else {
                    hi = g_h[cidx] - rq;
                    wi = g_w[cidx] - sq;
                    ok = ok && g_hr[cidx] == rr && g_wr[cidx] == sr;
                }
                ok = ok && (unsigned)hi < (unsigned)p.Hi && (unsigned)wi < (unsigned)p.Wi;
                b_reg[ps][cidx] = ok ? Elem<T>::load(in, g_base[cidx] + plane + hi * p.Wi + wi) : 0.0f;
            }
        }
    };

    auto store_slab = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps) {
            const int il = a_i + ps * A_RPP;
            if (il < BM) As[buf][a_kk * LDA + il] = a_reg[ps];
        }
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps)
#pragma unroll
            for (int cidx = 0; cidx < B_COLS; ++cidx)
                Bs[buf][(ps * B_RPP + b_row) * LDB + (tid % BN) + cidx * NT] = b_reg[ps][cidx];
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

    const int n_slabs = (p.Kg + BK - 1) / BK;
    load_slab(0);
    store_slab(0);
    __syncthreads();

    const int a_off = wm * TM * 32 + (lane & 31);
    const int b_off = wn * TN * 32 + (lane & 31);
    const int khalf = lane >> 5;

    for (int slab = 0; slab < n_slabs; ++slab) {
        const int buf = slab & 1;
        const bool more = slab + 1 < n_slabs;
        if (more) load_slab(slab + 1);   // global loads in flight while the MFMAs below run
#pragma unroll
        for (int ks = 0; ks < BK / 2; ++ks) {
            const int row = 2 * ks + khalf;
            float av[TM], bv[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a) av[a] = As[buf][row * LDA + a_off + a * 32];
#pragma unroll
            for (int b = 0; b < TN; ++b) bv[b] = Bs[buf][row * LDB + b_off + b * 32];
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[a], bv[b], acc[a][b], 0, 0, 0);
        }
        if (more) store_slab(buf ^ 1);
        __syncthreads();
    }

    // ---- epilogue: accumulator register e of a 32x32 tile holds row (e/4)*8 + (lane/32)*4 + e%4,
    //      column lane%32 ----
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int pix = j0 + b_off + b * 32;
        if (pix >= p.M) continue;
        const int n = fastdiv(pix, p.div_howo);
        const int rem = pix - n * p.HoWo;
        const int obase = n * p.Co * p.HoWo + rem;
#pragma unroll
        for (int a = 0; a < TM; ++a) {
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = i0 + wm * TM * 32 + a * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3);
                if (i < p.Co) {
                    const int o = obase + i * p.HoWo;
                    float v = acc[a][b][e];
                    if (p.beta != 0.0f) v += Elem<T>::load(out, o);
                    Elem<T>::store(out, o, v);
                }
            }
        }
    }
}

template <typename T, int MODE, int TM, int TN, int WM, int WN>
hipError_t launch_cfg(PixGemmParams& p, hipStream_t st) {
    constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
    p.tiles_i = (p.Co + BM - 1) / BM;
    p.tiles_pix = (p.M + BN - 1) / BN;
    const long long total = (long long)p.tiles_i * p.tiles_pix;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    hipLaunchKernelGGL((igemm_pix_kernel<T, MODE, TM, TN, WM, WN>), dim3((unsigned)total),
                       dim3(WM * WN * 64), 0, st, p);
    return hipGetLastError();
}

template <typename T, int MODE>
hipError_t dispatch_tile(PixGemmParams& p, hipStream_t st) {
    // Channel-tile extent: the candidate (128, 96, 64, 32) that wastes the fewest padded rows,
    // larger on ties. Pixel-tile extent: 256 while that still leaves >= 2 workgroups per CU.
    const int cands[4] = {128, 96, 64, 32};
    int bm = 32;
    long long best = -1;
    for (int c : cands) {
        const long long padded = (long long)((p.Co + c - 1) / c) * c;
        if (best < 0 || padded < best) { best = padded; bm = c; }
    }
    const long long tiles256 = (long long)((p.Co + bm - 1) / bm) * ((p.M + 255) / 256);
    const bool wide = tiles256 >= 512;
    switch (bm) {
        case 128: return launch_cfg<T, MODE, 2, 2, 2, 2>(p, st);
        case 96:  return wide ? launch_cfg<T, MODE, 3, 2, 1, 4>(p, st) : launch_cfg<T, MODE, 3, 1, 1, 4>(p, st);
        case 64:  return wide ? launch_cfg<T, MODE, 2, 2, 1, 4>(p, st) : launch_cfg<T, MODE, 2, 1, 1, 4>(p, st);
        default:  return wide ? launch_cfg<T, MODE, 1, 2, 1, 4>(p, st) : launch_cfg<T, MODE, 1, 1, 1, 4>(p, st);
    }
}

}  // namespace

hipError_t launch_conv_pix(bool bwd_data, int dtype, const ConvGeom& g, const void* in,
                           const void* wt, void* out, float beta, hipStream_t st) {
    if (bwd_data && conv_bwd_data_smallc_applies(g))
        return launch_conv_bwd_data_smallc(dtype, g, in, wt, out, beta, st);
    PixGemmParams p{};
    p.in = in; p.wt = wt; p.out = out;
    p.N = g.N;
    p.R = g.R; p.S = g.S; p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.RS = g.R * g.S;
    if (!bwd_data) {
        p.Ci = g.C; p.Hi = g.H; p.Wi = g.W;
        p.Co = g.K; p.Ho = g.P; p.Wo = g.Q;
        p.a_ci_stride = p.RS;            // w[k][c][rs]: i = k, ci = c
        p.a_i_stride = g.C * p.RS;
    } else {
        p.Ci = g.K; p.Hi = g.P; p.Wi = g.Q;
        p.Co = g.C; p.Ho = g.H; p.Wo = g.W;
        p.a_ci_stride = g.C * p.RS;      // w[k][c][rs]: i = c, ci = k
        p.a_i_stride = p.RS;
    }
    p.Kg = p.Ci * p.RS;
    p.HiWi = p.Hi * p.Wi;
    p.HoWo = p.Ho * p.Wo;
    p.M = p.N * p.HoWo;
    p.div_rs = make_fastdiv(p.RS);
    p.div_s = make_fastdiv(p.S);
    p.div_howo = make_fastdiv(p.HoWo);
    p.div_wo = make_fastdiv(p.Wo);
    p.div_sh = make_fastdiv(p.sh);
    p.div_sw = make_fastdiv(p.sw);
    p.beta = beta;
    if (dtype == PURINE_F32)
        return bwd_data ? dispatch_tile<float, 1>(p, st) : dispatch_tile<float, 0>(p, st);
    return bwd_data ? dispatch_tile<uint16_t, 1>(p, st) : dispatch_tile<uint16_t, 0>(p, st);
}

}  // namespace purine

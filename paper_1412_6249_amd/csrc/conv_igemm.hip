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

// MODE 0 = forward, MODE 1 = backward-data with unit stride, MODE 2 = backward-data with a stride
// (phase-folded, see launch_conv_pix). Workgroup = WM x WN wavefronts, each owning TM x TN MFMA
// tiles of 32 x 32.
template <typename T, int MODE, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void igemm_pix_kernel(const PixGemmParams p) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    constexpr int LDA = BM + 2;   // +2: the transposed filter-slab store hits distinct banks
    constexpr int LDB = BN;
    static_assert(NT % BN == 0 && NT >= BN, "one pixel column per thread");
    constexpr int B_RPP = NT / BN;       // slab rows covered per pass
    constexpr int B_PASSES = BK / B_RPP;
    static_assert(BK % B_RPP == 0, "row mapping");
    constexpr int A_RPP = NT / BK;       // filter rows (channels) per pass
    constexpr int A_PASSES = BM / A_RPP;
    static_assert(BM % A_RPP == 0, "filter mapping");

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

    // ---- this thread's pixel column of the patch slab (fixed for the whole kernel) ----
    // g_off: element offset of the tap (ci=0, r=0, s=0) of this pixel inside `in`; g_h/g_w: the
    // coordinates that the bounds test compares against.
    int g_off, g_h, g_w;
    bool g_live;
    {
        const int pix = j0 + (tid % BN);
        g_live = pix < p.M;
        const int pc = g_live ? pix : 0;
        const int n = fastdiv(pc, p.div_howo);
        const int rem = pc - n * p.HoWo;
        const int ho = fastdiv(rem, p.div_wo);
        const int wo = rem - ho * p.Wo;
        if (MODE == 0) { g_h = ho * p.sh - p.ph; g_w = wo * p.sw - p.pw; }   // hi = g_h + r
        else if (MODE == 1) { g_h = ho + p.ph; g_w = wo + p.pw; }            // hi = g_h - r
        else { g_h = ho + p.hq_min; g_w = wo + p.wq_min; }                   // hi = hq - r'
        g_off = n * p.Ci * p.HiWi + g_h * p.Wi + g_w;
    }
    const int b_row = __builtin_amdgcn_readfirstlane(tid / BN);  // uniform per wavefront (BN >= 64)
    const int a_kk = tid % BK;
    const int a_i = tid / BK;

    // ---- this thread's rows of the filter slab ----
    // a_base: offset of row i at (ci=0, r'=0, s'=0); MODE 2 also keeps the row's phase (a, b)
    int a_base[A_PASSES], a_ab[A_PASSES];
#pragma unroll
    for (int ps = 0; ps < A_PASSES; ++ps) {
        const int i = i0 + a_i + ps * A_RPP;
        if (i < p.Co) {
            if (MODE == 2) {
                const int c = fastdiv(i, p.div_phases);
                const int ab = i - c * p.phases;
                const int a = fastdiv(ab, p.div_sw);
                const int b = ab - a * p.sw;
                a_base[ps] = c * p.R * p.S + a * p.S + b;
                a_ab[ps] = (a << 16) | b;
            } else {
                a_base[ps] = i * p.a_i_stride;
                a_ab[ps] = 0;
            }
        } else {
            a_base[ps] = 0;
            a_ab[ps] = -1;
        }
    }

    // staged slab: raw loaded values plus one validity bit per value (the zero-fill select is
    // applied when the values go to LDS, so nothing forces an early wait on the loads)
    float a_reg[A_PASSES];
    float b_reg[B_PASSES];
    unsigned a_ok, b_ok;

    auto load_slab = [&](int slab) {
        a_ok = 0u; b_ok = 0u;
        // filter slab: A[i, kk] for kk = slab*BK + a_kk
        {
            const int kk = slab * BK + a_kk;
            const bool kv = kk < p.Kg;
            const int kq = kv ? kk : 0;
            const int ci = fastdiv(kq, p.div_rs);
            const int rs = kq - ci * p.RS;
            if (MODE == 2) {
                const int rp = fastdiv(rs, p.div_s);
                const int sp = rs - rp * p.Sp;
                const int r0 = rp * p.sh, s0 = sp * p.sw;     // tap of phase (0,0); row adds (a, b)
                const int off = ci * p.a_ci_stride + r0 * p.S + s0;
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps) {
                    const int a = a_ab[ps] >> 16, b = a_ab[ps] & 0xffff;
                    const bool ok = kv & (a_ab[ps] >= 0) & (r0 + a < p.R) & (s0 + b < p.S);
                    a_reg[ps] = Elem<T>::load(wt, ok ? off + a_base[ps] : 0);   // clamped, branch-free
                    a_ok |= (ok ? 1u : 0u) << ps;
                }
            } else {
                const int off = ci * p.a_ci_stride + rs;
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps) {
                    const bool ok = kv & (a_ab[ps] >= 0);
                    a_reg[ps] = Elem<T>::load(wt, ok ? off + a_base[ps] : 0);
                    a_ok |= (ok ? 1u : 0u) << ps;
                }
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
            const int s = rs - r * (MODE == 2 ? p.Sp : p.S);
            const int tap = r * p.Wi + s;
            int hi, wi, off;
            if (MODE == 0) { hi = g_h + r; wi = g_w + s; off = ci * p.HiWi + tap; }
            else           { hi = g_h - r; wi = g_w - s; off = ci * p.HiWi - tap; }
            // bitwise & on purpose: no short-circuit control flow inside the slab loop
            const bool ok = kv & g_live & ((unsigned)hi < (unsigned)p.Hi) & ((unsigned)wi < (unsigned)p.Wi);
            // clamped index instead of a predicated load: keeps the loop one basic block
            b_reg[ps] = Elem<T>::load(in, ok ? g_off + off : 0);
            b_ok |= (ok ? 1u : 0u) << ps;
        }
    };

    auto store_slab = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps)
            As[buf][a_kk * LDA + a_i + ps * A_RPP] = ((a_ok >> ps) & 1u) ? a_reg[ps] : 0.0f;
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps)
            Bs[buf][(ps * B_RPP + b_row) * LDB + (tid % BN)] = ((b_ok >> ps) & 1u) ? b_reg[ps] : 0.0f;
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
        load_slab(slab + 1);   // global loads in flight while the MFMAs below run (past the end: zeros)
        float av[2][TM], bv[2][TN];   // operand fragments, double-buffered across k-steps
#pragma unroll
        for (int a = 0; a < TM; ++a) av[0][a] = As[buf][khalf * LDA + a_off + a * 32];
#pragma unroll
        for (int b = 0; b < TN; ++b) bv[0][b] = Bs[buf][khalf * LDB + b_off + b * 32];
#pragma unroll
        for (int ks = 0; ks < BK / 2; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks + 1 < BK / 2) {
                const int row = 2 * (ks + 1) + khalf;
#pragma unroll
                for (int a = 0; a < TM; ++a) av[nxt][a] = As[buf][row * LDA + a_off + a * 32];
#pragma unroll
                for (int b = 0; b < TN; ++b) bv[nxt][b] = Bs[buf][row * LDB + b_off + b * 32];
            }
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][a], bv[cur][b], acc[a][b], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the zero-fill selects (and their load waits) below the MFMAs
        store_slab(buf ^ 1);
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
        if (MODE != 2) {
            const int obase = n * p.Co * p.HoWo + rem;
#pragma unroll
            for (int a = 0; a < TM; ++a)
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
        } else {
            // depth-to-space: row i = (c, a, b) of pixel (n, hq, wq) is dx[n, c, hq*sh+a-ph, wq*sw+b-pw]
            const int hq = fastdiv(rem, p.div_wo);
            const int wq = rem - hq * p.Wo;
            const int hb = (hq + p.hq_min) * p.sh - p.ph;
            const int wb = (wq + p.wq_min) * p.sw - p.pw;
            const int obase = n * p.C * p.H * p.W;
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int i = i0 + wm * TM * 32 + a * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3);
                    if (i < p.Co) {
                        const int c = fastdiv(i, p.div_phases);
                        const int ab = i - c * p.phases;
                        const int pa = fastdiv(ab, p.div_sw);
                        const int pb = ab - pa * p.sw;
                        const int h = hb + pa, w = wb + pb;
                        if ((unsigned)h < (unsigned)p.H && (unsigned)w < (unsigned)p.W) {
                            const int o = obase + (c * p.H + h) * p.W + w;
                            float v = acc[a][b][e];
                            if (p.beta != 0.0f) v += Elem<T>::load(out, o);
                            Elem<T>::store(out, o, v);
                        }
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
    PixGemmParams p{};
    p.in = in; p.wt = wt; p.out = out;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W;
    p.R = g.R; p.S = g.S; p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.RS = g.R * g.S;
    p.Sp = g.S;
    p.phases = 1;
    int mode = 0;
    if (!bwd_data) {
        p.Ci = g.C; p.Hi = g.H; p.Wi = g.W;
        p.Co = g.K; p.Ho = g.P; p.Wo = g.Q;
        p.a_ci_stride = p.RS;            // w[k][c][rs]: i = k, ci = c
        p.a_i_stride = g.C * p.RS;
    } else if (g.sh == 1 && g.sw == 1) {
        mode = 1;
        p.Ci = g.K; p.Hi = g.P; p.Wi = g.Q;
        p.Co = g.C; p.Ho = g.H; p.Wo = g.W;
        p.a_ci_stride = g.C * p.RS;      // w[k][c][rs]: i = c, ci = k
        p.a_i_stride = p.RS;
    } else {
        // Strided backward-data, phase-folded. Write h + ph = hq*sh + a and w + pw = wq*sw + b.
        // Only taps r = a + sh*r', s = b + sw*s' reach such a position, from p = hq - r',
        // q = wq - s'. So dx is a unit-stride correlation of dy with ceil(R/sh) x ceil(S/sw) taps that
        // produces C*sh*sw "channels" (c, a, b) per coarse pixel (hq, wq), followed by a
        // depth-to-space shuffle in the epilogue. No multiply is spent on the structural zeros of
        // the strided transposed convolution, and the GEMM's row count grows from C to C*sh*sw.
        mode = 2;
        p.Ci = g.K; p.Hi = g.P; p.Wi = g.Q;
        p.phases = g.sh * g.sw;
        p.Co = g.C * p.phases;
        p.hq_min = g.ph / g.sh;
        p.wq_min = g.pw / g.sw;
        p.Ho = (g.H - 1 + g.ph) / g.sh - p.hq_min + 1;
        p.Wo = (g.W - 1 + g.pw) / g.sw - p.wq_min + 1;
        const int Rp = (g.R + g.sh - 1) / g.sh;
        p.Sp = (g.S + g.sw - 1) / g.sw;
        p.RS = Rp * p.Sp;
        p.a_ci_stride = g.C * g.R * g.S;
        p.a_i_stride = 0;
    }
    p.Kg = p.Ci * p.RS;
    p.HiWi = p.Hi * p.Wi;
    p.HoWo = p.Ho * p.Wo;
    p.M = p.N * p.HoWo;
    p.div_rs = make_fastdiv(p.RS);
    p.div_s = make_fastdiv(mode == 2 ? p.Sp : p.S);
    p.div_howo = make_fastdiv(p.HoWo);
    p.div_wo = make_fastdiv(p.Wo);
    p.div_phases = make_fastdiv(p.phases);
    p.div_sw = make_fastdiv(p.sw);
    p.beta = beta;
    if (dtype == PURINE_F32) {
        if (mode == 0) return dispatch_tile<float, 0>(p, st);
        return mode == 1 ? dispatch_tile<float, 1>(p, st) : dispatch_tile<float, 2>(p, st);
    }
    if (mode == 0) return dispatch_tile<uint16_t, 0>(p, st);
    return mode == 1 ? dispatch_tile<uint16_t, 1>(p, st) : dispatch_tile<uint16_t, 2>(p, st);
}

}  // namespace purine

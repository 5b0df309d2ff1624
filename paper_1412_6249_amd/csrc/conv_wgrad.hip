// Weight-gradient implicit GEMM for gfx950 (the ConvBwdWeight operator of paper Figure 1(b)).
//
//     dw[k, (c,r,s)] = sum over pixels (n,p,q) of dy[n,k,p,q] * x[n,c,p*sh-ph+r,q*sw-pw+s]
//
// The reduction runs over all N*P*Q pixels while the output is tiny, so the pixel range is cut
// into `splits` chunks. Workgroup (tile, split) reduces its chunk on the fp32 MFMA units and
// writes an fp32 partial tile to scratch; a second kernel adds the partials in chunk order
// (fixed order: bit-identical run to run, no atomics). The split also bounds the length of any
// single fp32 accumulation chain, which the 1e-5 accuracy target needs for 10^5..10^6 pixels.
// Neither operand is materialised: both slabs are built in LDS from the NCHW tensors with lanes
// running along pixels.
#include "common.h"

namespace purine {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int BK = 16;  // pixels per slab

template <typename T> __device__ __forceinline__ float ld(const T* p, int i);
template <> __device__ __forceinline__ float ld<float>(const float* p, int i) { return p[i]; }
template <> __device__ __forceinline__ float ld<uint16_t>(const uint16_t* p, int i) {
    return __uint_as_float(((uint32_t)p[i]) << 16);
}

// tile extents -> (TM, TN, WM, WN); CALL3 serves the one tile of three wavefronts (fp32 only)
#define WGRAD_TILE_SWITCH(CALL, CALL3)                                           \
    switch (plan.bm * 1000 + plan.bn) {                                          \
        case 128128: return CALL(2, 2, 2, 2);                                    \
        case 96096:  return CALL3(3, 1, 1, 3);                                   \
        case 128096: return CALL(1, 3, 4, 1);                                    \
        case 192064: return CALL(3, 1, 2, 2);                                    \
        case 128064: return CALL(1, 2, 4, 1);                                    \
        case 96128:  return CALL(3, 1, 1, 4);                                    \
        case 64128:  return CALL(2, 1, 1, 4);                                    \
        case 64064:  return CALL(1, 1, 2, 2);                                    \
        case 32128:  return CALL(1, 1, 1, 4);                                    \
        default: return hipErrorInvalidValue;                                    \
    }

// Column modes of the output tile.
//   TAP = false: columns are the flattened (c, r, s) index; every column has its own tap, so every
//                gathered element carries its own bounds test (layers with few input channels).
//   TAP = true : the workgroup owns ONE tap (r, s) and its columns are input channels c. The bounds
//                test and the tap offset are then per pixel, once per slab, and a gathered element
//                is one add and one load. Partials are laid out [split][tap][k][c] (coalesced along
//                c); the reduction kernel writes them back in KCRS order.
struct TileWhere {
    int split, i0, j0, tap_r, tap_s, tap;
};
// Consecutive workgroup ids land on different XCDs (8 per chip, each with its own L2). The tiles of
// one split read the same chunk of x and dy, so each XCD gets a contiguous run of (split, tile) ids:
// a chunk is then fetched into one L2 instead of all eight.
__device__ __forceinline__ int xcd_run(int bid, int total) {
    const int per = total >> 3;
    return (per > 0 && bid < per * 8) ? (bid & 7) * per + (bid >> 3) : bid;
}
template <bool TAP, int BM, int BN>
__device__ __forceinline__ TileWhere locate_tile(const WgradParams& p) {
    TileWhere t;
    int bid = xcd_run(blockIdx.x, gridDim.x);
    const int per_split = p.tiles_i * p.tiles_j;
    t.split = bid / per_split;
    bid -= t.split * per_split;
    t.i0 = (bid % p.tiles_i) * BM;
    const int jt = bid / p.tiles_i;
    if (TAP) {
        t.tap = jt / p.c_tiles;
        t.j0 = (jt - t.tap * p.c_tiles) * BN;
        t.tap_r = fastdiv(t.tap, p.div_s);
        t.tap_s = t.tap - t.tap_r * p.S;
    } else {
        t.tap = t.tap_r = t.tap_s = 0;
        t.j0 = jt * BN;
    }
    return t;
}

// BUF: both operands are read with raw buffer loads, whose hardware range check returns zero for a
// byte offset at or beyond the tensor's size. A thread's offset is the sum of a per-slab pixel part
// (2^31 when the pixel does not exist or, per-tap mode, its tap falls outside the image) and a
// per-row part fixed for the kernel (2^30 when the row or column does not exist); the host enables
// BUF for tensors below 2^30 bytes, so every such sum is out of range without wrapping, and the slab
// loop needs no clamped addresses, validity bits or zero-fill selects. NOPAD (flattened columns of
// an unpadded layer): every tap of an existing pixel is inside the image, so the flattened mode
// gets the same two-part offsets.
template <typename T, bool TAP, bool NOPAD, bool BUF, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void wgrad_kernel(const WgradParams p) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;   // output channels k
    constexpr int BN = WN * TN * 32;   // columns: (c,r,s) flattened, or channels of one tap
    constexpr int LDA = BM + 2, LDB = BN + 2;
    constexpr int RPP = NT / BK;       // tile columns covered per pass (lanes 0..15 run along pixels)
    constexpr int A_PASSES = BM / RPP, B_PASSES = BN / RPP;
    static_assert(BM % RPP == 0 && BN % RPP == 0, "mapping");

    __shared__ float As[2][BK * LDA];
    __shared__ float Bs[2][BK * LDB];

    const T* __restrict__ x = (const T*)p.x;
    const T* __restrict__ dy = (const T*)p.dy;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const TileWhere tw = locate_tile<TAP, BM, BN>(p);
    const int i0 = tw.i0, j0 = tw.j0;
    const int pix_begin = tw.split * p.chunk;
    const int pix_end = min(p.M, pix_begin + p.chunk);

    const int t_kk = tid % BK;   // this thread's pixel inside a slab
    const int t_col = tid / BK;  // first tile column it serves

    // columns served by this thread: fixed for the whole kernel
    int j_off[B_PASSES], j_rs[B_PASSES];
#pragma unroll
    for (int ps = 0; ps < B_PASSES; ++ps) {
        const int j = j0 + t_col + ps * RPP;
        if (TAP) {
            j_off[ps] = j * p.HW;
            j_rs[ps] = j < p.C ? 0 : -1;
        } else if (j < p.CRS) {
            const int c = fastdiv(j, p.div_rs);
            const int rs = j - c * p.RS;
            const int r = fastdiv(rs, p.div_s);
            const int s = rs - r * p.S;
            j_off[ps] = c * p.HW + r * p.W + s;
            j_rs[ps] = (r << 16) | s;
        } else {
            j_off[ps] = 0;
            j_rs[ps] = -1;
        }
    }

    float a_reg[A_PASSES], b_reg[B_PASSES];
    unsigned a_ok = 0u, b_ok = 0u;   // validity bits; the zero-fill happens at the LDS store

    constexpr bool B_TWO_PART = BUF && (TAP || NOPAD);   // x offsets split into pixel part + column part
    const __amdgpu_buffer_rsrc_t rs_dy =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(dy), (short)0, BUF ? (int)p.dy_bytes : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(x), (short)0, BUF ? (int)p.x_bytes : 0, 0x00020000);
    // per-row / per-column byte offsets, fixed for the kernel
    unsigned a_voff[BUF ? A_PASSES : 1], b_voff[B_TWO_PART ? B_PASSES : 1];
    if (BUF) {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps) {
            const int i = i0 + t_col + ps * RPP;
            a_voff[BUF ? ps : 0] = i < p.K ? (unsigned)(i * p.PQ) * 4u : 0x40000000u;
        }
    }
    if (B_TWO_PART) {
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps)
            b_voff[B_TWO_PART ? ps : 0] = j_rs[ps] >= 0 ? (unsigned)j_off[ps] * 4u : 0x40000000u;
    }

    auto load_slab = [&](int slab) {
        const int pix = pix_begin + slab * BK + t_kk;
        const bool pv = pix < pix_end;
        const int pc = pv ? pix : 0;
        const int n = fastdiv(pc, p.div_pq);
        const int pq = pc - n * p.PQ;
        const int pp = fastdiv(pq, p.div_q);
        const int qq = pq - pp * p.Q;
        const int a_base = n * p.dy_ns + pq;
        a_ok = 0u; b_ok = 0u;
        if (BUF) {
            const unsigned a_pix = pv ? (unsigned)a_base * 4u : 0x80000000u;
#pragma unroll
            for (int ps = 0; ps < A_PASSES; ++ps)
                a_reg[ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_dy, a_pix + a_voff[BUF ? ps : 0], 0, 0));
        } else {
#pragma unroll
            for (int ps = 0; ps < A_PASSES; ++ps) {
                const int i = i0 + t_col + ps * RPP;
                const bool ok = pv & (i < p.K);
                a_reg[ps] = ld<T>(dy, ok ? a_base + i * p.PQ : 0);   // clamped, branch-free
                a_ok |= (ok ? 1u : 0u) << ps;
            }
        }
        const int hb = pp * p.sh - p.ph + tw.tap_r, wb = qq * p.sw - p.pw + tw.tap_s;
        const int b_base = n * p.x_ns + hb * p.W + wb;
        if (B_TWO_PART) {
            // per-tap mode: one bounds test for the pixel's tap; unpadded flattened mode: none
            const bool in = TAP ? (pv & ((unsigned)hb < (unsigned)p.H) & ((unsigned)wb < (unsigned)p.W)) : pv;
            const unsigned b_pix = in ? (unsigned)b_base * 4u : 0x80000000u;
#pragma unroll
            for (int ps = 0; ps < B_PASSES; ++ps)
                b_reg[ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_x, b_pix + b_voff[B_TWO_PART ? ps : 0], 0, 0));
        } else if (TAP) {
            const bool in = pv & ((unsigned)hb < (unsigned)p.H) & ((unsigned)wb < (unsigned)p.W);
#pragma unroll
            for (int ps = 0; ps < B_PASSES; ++ps) {
                const bool ok = in & (j_rs[ps] >= 0);
                b_reg[ps] = ld<T>(x, ok ? b_base + j_off[ps] : 0);
                b_ok |= (ok ? 1u : 0u) << ps;
            }
        } else {
#pragma unroll
            for (int ps = 0; ps < B_PASSES; ++ps) {
                const int r = j_rs[ps] >> 16, s = j_rs[ps] & 0xffff;
                const bool ok = pv & (j_rs[ps] >= 0) & ((unsigned)(hb + r) < (unsigned)p.H) &
                                ((unsigned)(wb + s) < (unsigned)p.W);
                if (BUF) {
                    b_reg[ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(
                        rs_x, ok ? (unsigned)(b_base + j_off[ps]) * 4u : 0x80000000u, 0, 0));
                } else {
                    b_reg[ps] = ld<T>(x, ok ? b_base + j_off[ps] : 0);
                    b_ok |= (ok ? 1u : 0u) << ps;
                }
            }
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps)
            As[buf][t_kk * LDA + t_col + ps * RPP] = (BUF || ((a_ok >> ps) & 1u)) ? a_reg[ps] : 0.0f;
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps)
            Bs[buf][t_kk * LDB + t_col + ps * RPP] = (BUF || ((b_ok >> ps) & 1u)) ? b_reg[ps] : 0.0f;
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;
    // Fused bias gradient: the dy fragments that feed the MFMAs are also summed per lane (one add per
    // fragment; masked pixels and rows are zeros in LDS). Only the wavefronts that hold the first
    // column block of the first column tile write their sums, so every (split, k) is written once.
    float dbacc[TM];
#pragma unroll
    for (int a = 0; a < TM; ++a) dbacc[a] = 0.0f;
    const bool do_db = p.db_out != nullptr && j0 == 0 && tw.tap == 0 && wn == 0;

    const int n_slabs = (pix_end - pix_begin + BK - 1) / BK;   // >= 0; zero slabs leave zeros
    if (n_slabs > 0) {
        load_slab(0);
        store_slab(0);
    }
    __syncthreads();

    const int a_off = wm * TM * 32 + (lane & 31);
    const int b_off = wn * TN * 32 + (lane & 31);
    const int khalf = lane >> 5;

    for (int slab = 0; slab < n_slabs; ++slab) {
        const int buf = slab & 1;
        load_slab(slab + 1);   // past the chunk: every value is masked to zero
        __builtin_amdgcn_sched_barrier(0);   // the loads stay ahead of this slab's MFMAs
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
#pragma unroll
            for (int a = 0; a < TM; ++a) dbacc[a] += av[cur][a];
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the LDS stores (and their load waits) below the MFMAs
        store_slab(buf ^ 1);
        __syncthreads();
    }

    // partial tile: [split][k][(c,r,s)] or, per tap, [split][tap][k][c]
    const int ncol = TAP ? p.C : p.CRS;
    float* __restrict__ out = p.out + (size_t)tw.split * p.K * p.CRS + (TAP ? (size_t)tw.tap * p.K * p.C : 0);
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int j = j0 + b_off + b * 32;
        if (j >= ncol) continue;
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = i0 + wm * TM * 32 + a * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3);
                if (i < p.K) out[(size_t)i * ncol + j] = acc[a][b][e];
            }
    }
    if (do_db) {   // wavefront-uniform: lanes l and l+32 hold the even and odd pixels of row l
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const float tot = dbacc[a] + __shfl_xor(dbacc[a], 32);
            const int i = i0 + wm * TM * 32 + a * 32 + (lane & 31);
            if (khalf == 0 && i < p.K) p.db_out[(size_t)tw.split * p.K + i] = tot;
        }
    }
}

// sum of the eight bf16 values of an MFMA operand fragment, in a fixed order
__device__ __forceinline__ float sum8(const uint4 u) {
    const float s0 = __uint_as_float(u.x << 16) + __uint_as_float(u.x & 0xffff0000u);
    const float s1 = __uint_as_float(u.y << 16) + __uint_as_float(u.y & 0xffff0000u);
    const float s2 = __uint_as_float(u.z << 16) + __uint_as_float(u.z & 0xffff0000u);
    const float s3 = __uint_as_float(u.w << 16) + __uint_as_float(u.w & 0xffff0000u);
    return (s0 + s1) + (s2 + s3);
}

// ------------------------------------------------------------------------------------------------
// bf16 MFMA variant (v_mfma_f32_32x32x16_bf16): the reduction runs over pixels, and NCHW keeps the
// pixels of one channel contiguous, so both operands are reduction-major already: the LDS tiles are
// As[k][pixel] and Bs[(c,r,s)][pixel] with a slab of 32 pixels, rows padded to 40 elements so the
// 16-byte fragment reads of 32 rows fall in distinct bank groups. VEC_A: a slab never straddles an
// image and stays 16-byte aligned (P*Q a multiple of 32), so dy rows are read with 16-byte loads.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
constexpr int BKP = 32;
constexpr int LDP = BKP + 8;

// BUF / NOPAD as in the fp32 kernel: the gathered x elements (and dy, when it is read element by
// element) come through raw buffer loads with two-part byte offsets, zeros from the range check.
template <bool VEC_A, bool TAP, bool NOPAD, bool BUF, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void wgrad_bf16_kernel(const WgradParams p) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    constexpr int RPP = NT / BKP;      // tile rows covered per pass (lanes 0..31 run along pixels)
    constexpr int A_PASSES = BM / RPP, B_PASSES = BN / RPP;
    constexpr int A_VEC = BM * (BKP / 8);
    constexpr int A_ITERS = (A_VEC + NT - 1) / NT;
    static_assert(NT == 256 && BM % RPP == 0 && BN % RPP == 0, "mapping");

    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDP];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDP];

    const uint16_t* __restrict__ x = (const uint16_t*)p.x;
    const uint16_t* __restrict__ dy = (const uint16_t*)p.dy;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const TileWhere tw = locate_tile<TAP, BM, BN>(p);
    const int split = tw.split, i0 = tw.i0, j0 = tw.j0;
    const int pix_begin = split * p.chunk;
    const int pix_end = min(p.M, pix_begin + p.chunk);

    const int t_px = tid % BKP;   // this thread's pixel inside a slab
    const int t_row = tid / BKP;  // first tile row it serves

    int j_off[B_PASSES], j_rs[B_PASSES];
#pragma unroll
    for (int ps = 0; ps < B_PASSES; ++ps) {
        const int j = j0 + t_row + ps * RPP;
        if (TAP) {
            j_off[ps] = j * p.HW;
            j_rs[ps] = j < p.C ? 0 : -1;
        } else if (j < p.CRS) {
            const int c = fastdiv(j, p.div_rs);
            const int rs = j - c * p.RS;
            const int r = fastdiv(rs, p.div_s);
            const int s = rs - r * p.S;
            j_off[ps] = c * p.HW + r * p.W + s;
            j_rs[ps] = (r << 16) | s;
        } else {
            j_off[ps] = 0;
            j_rs[ps] = -1;
        }
    }

    uint32_t a_reg[VEC_A ? 1 : A_PASSES];
    uint4 a_vec[VEC_A ? A_ITERS : 1];
    uint32_t b_reg[B_PASSES];
    unsigned a_ok = 0u, b_ok = 0u;

    constexpr bool A_BUF = BUF && !VEC_A;
    constexpr bool B_TWO_PART = BUF && (TAP || NOPAD);
    const __amdgpu_buffer_rsrc_t rs_dy =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(dy), (short)0, BUF ? (int)p.dy_bytes : 0, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(x), (short)0, BUF ? (int)p.x_bytes : 0, 0x00020000);
    unsigned a_voff[A_BUF ? A_PASSES : 1], b_voff[B_TWO_PART ? B_PASSES : 1];
    if (A_BUF) {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps) {
            const int i = i0 + t_row + ps * RPP;
            a_voff[A_BUF ? ps : 0] = i < p.K ? (unsigned)(i * p.PQ) * 2u : 0x40000000u;
        }
    }
    if (B_TWO_PART) {
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps)
            b_voff[B_TWO_PART ? ps : 0] = j_rs[ps] >= 0 ? (unsigned)j_off[ps] * 2u : 0x40000000u;
    }

    auto load_slab = [&](int slab) {
        const int pix0 = pix_begin + slab * BKP;
        const int pix = pix0 + t_px;
        const bool pv = pix < pix_end;
        const int pc = pv ? pix : 0;
        const int n = fastdiv(pc, p.div_pq);
        const int pq = pc - n * p.PQ;
        const int pp = fastdiv(pq, p.div_q);
        const int qq = pq - pp * p.Q;
        if (VEC_A) {
            // whole slab inside one image: n0/pq0 are uniform; pixels past pix_end are masked at the store
            const int n0 = fastdiv(pix0 < p.M ? pix0 : 0, p.div_pq);
            const int pq0 = (pix0 < p.M ? pix0 : 0) - n0 * p.PQ;
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it) {
                const int f = tid + it * NT;
                const int row = f / (BKP / 8), piece = f - row * (BKP / 8);
                const bool ok = (f < A_VEC) & (i0 + row < p.K) & (pix0 + piece * 8 < pix_end);
                a_vec[it] = *reinterpret_cast<const uint4*>(
                    dy + (ok ? n0 * p.dy_ns + (i0 + row) * p.PQ + pq0 + piece * 8 : 0));
                a_ok = ok ? (a_ok | (1u << it)) : (a_ok & ~(1u << it));
            }
        } else {
            a_ok = 0u;
            const int a_base = n * p.dy_ns + pq;
            if (A_BUF) {
                const unsigned a_pix = pv ? (unsigned)a_base * 2u : 0x80000000u;
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps)
                    a_reg[ps] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs_dy, a_pix + a_voff[A_BUF ? ps : 0], 0, 0);
            } else {
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps) {
                    const int i = i0 + t_row + ps * RPP;
                    const bool ok = pv & (i < p.K);
                    a_reg[ps] = dy[ok ? a_base + i * p.PQ : 0];
                    a_ok |= (ok ? 1u : 0u) << ps;
                }
            }
        }
        b_ok = 0u;
        const int hb = pp * p.sh - p.ph + tw.tap_r, wb = qq * p.sw - p.pw + tw.tap_s;
        const int b_base = n * p.x_ns + hb * p.W + wb;
        const bool in = pv & ((unsigned)hb < (unsigned)p.H) & ((unsigned)wb < (unsigned)p.W);
        if (B_TWO_PART) {
            const unsigned b_pix = (TAP ? in : pv) ? (unsigned)b_base * 2u : 0x80000000u;
#pragma unroll
            for (int ps = 0; ps < B_PASSES; ++ps)
                b_reg[ps] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(rs_x, b_pix + b_voff[B_TWO_PART ? ps : 0], 0, 0);
            return;
        }
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps) {
            bool ok;
            if (TAP) {
                ok = in & (j_rs[ps] >= 0);
            } else {
                const int r = j_rs[ps] >> 16, s = j_rs[ps] & 0xffff;
                ok = pv & (j_rs[ps] >= 0) & ((unsigned)(hb + r) < (unsigned)p.H) &
                     ((unsigned)(wb + s) < (unsigned)p.W);
            }
            if (BUF) {
                b_reg[ps] = (uint16_t)__builtin_amdgcn_raw_buffer_load_b16(
                    rs_x, ok ? (unsigned)(b_base + j_off[ps]) * 2u : 0x80000000u, 0, 0);
            } else {
                b_reg[ps] = x[ok ? b_base + j_off[ps] : 0];
                b_ok |= (ok ? 1u : 0u) << ps;
            }
        }
    };
    auto store_slab = [&](int buf) {
        if (VEC_A) {
#pragma unroll
            for (int it = 0; it < A_ITERS; ++it) {
                const int f = tid + it * NT;
                const int row = f / (BKP / 8), piece = f - row * (BKP / 8);
                if (f < A_VEC)
                    *reinterpret_cast<uint4*>(&As[buf][row * LDP + piece * 8]) =
                        ((a_ok >> it) & 1u) ? a_vec[it] : make_uint4(0u, 0u, 0u, 0u);
            }
        } else {
#pragma unroll
            for (int ps = 0; ps < A_PASSES; ++ps)
                As[buf][(t_row + ps * RPP) * LDP + t_px] = (A_BUF || ((a_ok >> ps) & 1u)) ? (uint16_t)a_reg[ps] : (uint16_t)0;
        }
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps)
            Bs[buf][(t_row + ps * RPP) * LDP + t_px] = (BUF || ((b_ok >> ps) & 1u)) ? (uint16_t)b_reg[ps] : (uint16_t)0;
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;
    // fused bias gradient as in the fp32 kernel; here summing a fragment costs 16 VALU operations, so
    // only the wavefronts that write the sums (do_db is uniform over a wavefront) take it
    float dbacc[TM];
#pragma unroll
    for (int a = 0; a < TM; ++a) dbacc[a] = 0.0f;
    const bool do_db = p.db_out != nullptr && j0 == 0 && tw.tap == 0 && wn == 0;

    const int n_slabs = (pix_end - pix_begin + BKP - 1) / BKP;
    if (n_slabs > 0) {
        load_slab(0);
        store_slab(0);
    }
    __syncthreads();

    const int a_row = (wm * TM * 32 + (lane & 31)) * LDP + (lane >> 5) * 8;
    const int b_row = (wn * TN * 32 + (lane & 31)) * LDP + (lane >> 5) * 8;
    const int khalf = lane >> 5;

    for (int slab = 0; slab < n_slabs; ++slab) {
        const int buf = slab & 1;
        load_slab(slab + 1);   // past the chunk: every value is masked to zero
#pragma unroll
        for (int ks = 0; ks < BKP / 16; ++ks) {
            bf16x8 av[TM], bv[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a)
                av[a] = *reinterpret_cast<const bf16x8*>(&As[buf][a_row + a * 32 * LDP + ks * 16]);
#pragma unroll
            for (int b = 0; b < TN; ++b)
                bv[b] = *reinterpret_cast<const bf16x8*>(&Bs[buf][b_row + b * 32 * LDP + ks * 16]);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[a], bv[b], acc[a][b], 0, 0, 0);
            if (do_db) {
#pragma unroll
                for (int a = 0; a < TM; ++a) dbacc[a] += sum8(__builtin_bit_cast(uint4, av[a]));
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        store_slab(buf ^ 1);
        __syncthreads();
    }

    const int ncol = TAP ? p.C : p.CRS;
    float* __restrict__ out = p.out + (size_t)split * p.K * p.CRS + (TAP ? (size_t)tw.tap * p.K * p.C : 0);
    const int jb = j0 + wn * TN * 32 + (lane & 31);
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int j = jb + b * 32;
        if (j >= ncol) continue;
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int i = i0 + wm * TM * 32 + a * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3);
                if (i < p.K) out[(size_t)i * ncol + j] = acc[a][b][e];
            }
    }
    if (do_db) {   // lanes l and l+32 hold the two 8-pixel halves of row l's 16-pixel steps
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const float tot = dbacc[a] + __shfl_xor(dbacc[a], 32);
            const int i = i0 + wm * TM * 32 + a * 32 + (lane & 31);
            if (khalf == 0 && i < p.K) p.db_out[(size_t)split * p.K + i] = tot;
        }
    }
}

template <bool VEC_A, bool TAP, bool NOPAD, bool BUF, int TM, int TN, int WM, int WN>
hipError_t launch_tile_bf16(WgradParams& p, hipStream_t st) {
    const long long total = (long long)p.tiles_i * p.tiles_j * p.splits;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    hipLaunchKernelGGL((wgrad_bf16_kernel<VEC_A, TAP, NOPAD, BUF, TM, TN, WM, WN>), dim3((unsigned)total),
                       dim3(WM * WN * 64), 0, st, p);
    return hipGetLastError();
}

template <bool VEC_A, bool TAP, bool NOPAD, bool BUF>
hipError_t dispatch_bf16_mode(WgradParams& p, const WgradPlan& plan, hipStream_t st) {
#define CALL(TM, TN, WM, WN) launch_tile_bf16<VEC_A, TAP, NOPAD, BUF, TM, TN, WM, WN>(p, st)
#define CALL3(TM, TN, WM, WN) hipErrorInvalidValue   // the plan gives bf16 layers no such tile
    WGRAD_TILE_SWITCH(CALL, CALL3)
#undef CALL3
#undef CALL
}
template <bool VEC_A, bool TAP>
hipError_t dispatch_bf16(WgradParams& p, const WgradPlan& plan, hipStream_t st) {
    // measured: 2-byte buffer loads are 6-10 % faster than plain loads in every mode (the per-tap
    // mode with several taps only since a split's tiles share one XCD's L2)
    const bool buf = p.x_bytes != 0 && p.dy_bytes != 0;
    const bool nopad = !TAP && p.ph == 0 && p.pw == 0 && (p.P - 1) * p.sh + p.R <= p.H && (p.Q - 1) * p.sw + p.S <= p.W;
    if (!buf) return dispatch_bf16_mode<VEC_A, TAP, false, false>(p, plan, st);
    if (TAP) return dispatch_bf16_mode<VEC_A, TAP, false, true>(p, plan, st);
    return nopad ? dispatch_bf16_mode<VEC_A, false, true, true>(p, plan, st)
                 : dispatch_bf16_mode<VEC_A, false, false, true>(p, plan, st);
}

// dw[i] = beta*dw[i] + partial[0][i] + partial[1][i] + ... summed in a fixed tree: a workgroup owns
// 16 consecutive elements; each of its 16 "split lanes" adds the partials s = lane, lane+16, ... in
// order (independent loads, so many are in flight), and the 16 lane sums are then added in lane
// order through LDS. The order never depends on timing, so the result is bit-identical run to run.
// Workgroups past dw_blocks do the same for the fused bias gradient: partials [split][K] into db[K].
__global__ __launch_bounds__(256) void wgrad_reduce_kernel(const float* __restrict__ partial,
                                                           float* __restrict__ dw, int n,
                                                           int splits, float beta, int tap_major,
                                                           int K, int C, int RS, int dw_blocks,
                                                           const float* __restrict__ db_partial,
                                                           float* __restrict__ db) {
    __shared__ float red[16][17];
    const int e = threadIdx.x & 15, sl = threadIdx.x >> 4;
    int blk = blockIdx.x;
    if (blk >= dw_blocks) {   // uniform over the workgroup
        blk -= dw_blocks;
        partial = db_partial; dw = db; n = K; tap_major = 0;
    }
    const int i = blk * 16 + e;      // index in the partials' own order (coalesced reads)
    float acc = 0.0f;
    if (i < n) {
        int s = sl;
        for (; s + 48 < splits; s += 64) {
            const float v0 = partial[(size_t)s * n + i];
            const float v1 = partial[(size_t)(s + 16) * n + i];
            const float v2 = partial[(size_t)(s + 32) * n + i];
            const float v3 = partial[(size_t)(s + 48) * n + i];
            acc += v0; acc += v1; acc += v2; acc += v3;
        }
        for (; s < splits; s += 16) acc += partial[(size_t)s * n + i];
    }
    red[sl][e] = acc;
    __syncthreads();
    if (sl == 0 && i < n) {
        int dst = i;
        if (tap_major) {   // partials are [tap][k][c]; dw is [k][c][tap]
            const int tap = i / (K * C);
            const int kc = i - tap * (K * C);
            dst = kc * RS + tap;
        }
        float t = beta != 0.0f ? dw[dst] : 0.0f;
#pragma unroll
        for (int l = 0; l < 16; ++l) t += red[l][e];
        dw[dst] = t;
    }
}

// The same reduction for n a multiple of 4 (rows of the partials 16-byte aligned): a workgroup owns
// 32 consecutive elements (one 128-byte line per split, so no line is fetched by two workgroups on
// different L2s), 8 lanes x 16 bytes wide, and 32 split lanes deep; the 32 lane sums are added in
// lane order. Also a fixed order; which of the two kernels adds dw's partials depends on K*C*R*S
// alone, so ConvBwdWeight and the fused ConvBwdWeight+BiasBwd give the same bits for dw.
__global__ __launch_bounds__(256) void wgrad_reduce_vec_kernel(const float* __restrict__ partial,
                                                               float* __restrict__ dw, int n,
                                                               int splits, float beta, int tap_major,
                                                               int K, int C, int RS, int dw_blocks,
                                                               const float* __restrict__ db_partial,
                                                               float* __restrict__ db) {
    __shared__ float red[32][33];
    const int e4 = threadIdx.x & 7, sl = threadIdx.x >> 3;
    int blk = blockIdx.x;
    if (blk >= dw_blocks) {   // uniform over the workgroup: the fused bias gradient's partials
        blk -= dw_blocks;
        partial = db_partial; dw = db; n = K; tap_major = 0;
    }
    if (n & 3) {
        // bias-gradient partials of a layer whose K is not a multiple of 4 (rows not 16-byte aligned):
        // element by element, 32 elements x 8 split lanes; the rows of `red` the lanes do not fill
        // hold zeros, so the final sum below serves both forms
        const int e = threadIdx.x & 31, sl8 = threadIdx.x >> 5;
        const int j = blk * 32 + e;
        float a = 0.0f;
        if (j < n)
            for (int s = sl8; s < splits; s += 8) a += partial[(size_t)s * n + j];
#pragma unroll
        for (int r = 0; r < 4; ++r) red[sl8 + 8 * r][e] = r == 0 ? a : 0.0f;
        __syncthreads();
        if (sl8 == 0 && j < n) {
            float t = beta != 0.0f ? dw[j] : 0.0f;
#pragma unroll
            for (int l = 0; l < 32; ++l) t += red[l][e];
            dw[j] = t;
        }
        return;
    }
    const int i = blk * 32 + e4 * 4;
    float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    if (i < n) {   // n and i are multiples of 4: the whole packet exists
        int s = sl;
        for (; s + 96 < splits; s += 128) {
            const float4 v0 = *reinterpret_cast<const float4*>(partial + (size_t)s * n + i);
            const float4 v1 = *reinterpret_cast<const float4*>(partial + (size_t)(s + 32) * n + i);
            const float4 v2 = *reinterpret_cast<const float4*>(partial + (size_t)(s + 64) * n + i);
            const float4 v3 = *reinterpret_cast<const float4*>(partial + (size_t)(s + 96) * n + i);
            acc.x += v0.x; acc.y += v0.y; acc.z += v0.z; acc.w += v0.w;
            acc.x += v1.x; acc.y += v1.y; acc.z += v1.z; acc.w += v1.w;
            acc.x += v2.x; acc.y += v2.y; acc.z += v2.z; acc.w += v2.w;
            acc.x += v3.x; acc.y += v3.y; acc.z += v3.z; acc.w += v3.w;
        }
        for (; s < splits; s += 32) {
            const float4 v = *reinterpret_cast<const float4*>(partial + (size_t)s * n + i);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    }
    red[sl][e4 * 4 + 0] = acc.x; red[sl][e4 * 4 + 1] = acc.y;
    red[sl][e4 * 4 + 2] = acc.z; red[sl][e4 * 4 + 3] = acc.w;
    __syncthreads();
    const int e = threadIdx.x;
    const int j = blk * 32 + e;
    if (e < 32 && j < n) {
        int dst = j;
        if (tap_major) {   // partials are [tap][k][c]; dw is [k][c][tap]
            const int tap = j / (K * C);
            const int kc = j - tap * (K * C);
            dst = kc * RS + tap;
        }
        float t = beta != 0.0f ? dw[dst] : 0.0f;
#pragma unroll
        for (int l = 0; l < 32; ++l) t += red[l][e];
        dw[dst] = t;
    }
}

template <typename T, bool TAP, bool NOPAD, bool BUF, int TM, int TN, int WM, int WN>
hipError_t launch_tile(WgradParams& p, hipStream_t st) {
    const long long total = (long long)p.tiles_i * p.tiles_j * p.splits;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    hipLaunchKernelGGL((wgrad_kernel<T, TAP, NOPAD, BUF, TM, TN, WM, WN>), dim3((unsigned)total), dim3(WM * WN * 64),
                       0, st, p);
    return hipGetLastError();
}

template <bool TAP, bool NOPAD, bool BUF>
hipError_t dispatch_f32_mode(WgradParams& p, const WgradPlan& plan, hipStream_t st) {
#define CALL(TM, TN, WM, WN) launch_tile<float, TAP, NOPAD, BUF, TM, TN, WM, WN>(p, st)
    WGRAD_TILE_SWITCH(CALL, CALL)
#undef CALL
}
template <bool TAP>
hipError_t dispatch_f32(WgradParams& p, const WgradPlan& plan, hipStream_t st) {
    const bool buf = p.x_bytes != 0 && p.dy_bytes != 0;
    // unpadded layer: every tap of every output pixel lies inside the image
    const bool nopad = !TAP && p.ph == 0 && p.pw == 0 && (p.P - 1) * p.sh + p.R <= p.H && (p.Q - 1) * p.sw + p.S <= p.W;
    if (TAP) return buf ? dispatch_f32_mode<TAP, false, true>(p, plan, st) : dispatch_f32_mode<TAP, false, false>(p, plan, st);
    if (!buf) return dispatch_f32_mode<false, false, false>(p, plan, st);
    return nopad ? dispatch_f32_mode<false, true, true>(p, plan, st) : dispatch_f32_mode<false, false, true>(p, plan, st);
}

}  // namespace

WgradPlan plan_wgrad(const ConvGeom& g, int dtype) {
    WgradPlan pl{};
    {
        // bf16 3x3 / stride 1 / pad 1 layers with rows of whole 16-byte packets: operands staged in
        // LDS row by row, persistent workgroups (conv_wgrad_rows_bf16.hip); one partial tile per worker
        int workers = 0;
        if (dtype == PURINE_BF16 && !buffer_loads_disabled() && wgrad_rows_bf16_applies(g, &workers)) {
            pl.rows = true;
            pl.tap = true;          // partials are [split][tap][k][c], as in the per-tap mode
            pl.splits = workers;
            pl.bm = 64; pl.bn = 64; pl.tiles_i = (g.K + 63) / 64; pl.c_tiles = (g.C + 63) / 64; pl.tiles_j = 9 * pl.c_tiles;
            pl.chunk = 0;
            pl.ws_bytes = (size_t)workers * (size_t)g.K * (size_t)g.C * 9 * sizeof(float);
            pl.db_ws_bytes = (size_t)workers * (size_t)g.K * sizeof(float);
            return pl;
        }
        // bf16 layers with at most 160 filter elements per output channel (the first layer of an image
        // network): every wavefront holds the whole filter tile and the wavefronts split the pixels
        // (conv_wgrad_cols_bf16.hip); partials are [worker][k][c][r][s]
        const bool taps = dtype == PURINE_BF16 && !buffer_loads_disabled() && wgrad_taps_bf16_applies(g, &workers);
        if (taps || (dtype == PURINE_BF16 && !buffer_loads_disabled() && wgrad_cols_bf16_applies(g, &workers))) {
            // (at most 32 (c, r) pairs and a filter row shape the tap kernel is built for: one accumulator
            // tile per column tap, conv_wgrad_taps_bf16.hip; same layout of the partials)
            pl.taps = taps;
            pl.cols = !taps;
            pl.tap = false;
            pl.splits = workers;
            pl.bm = 64; pl.bn = 160; pl.tiles_i = (g.K + 63) / 64; pl.c_tiles = 0; pl.tiles_j = 1;
            pl.chunk = 0;
            pl.ws_bytes = (size_t)workers * (size_t)g.K * (size_t)g.C * g.R * g.S * sizeof(float);
            pl.db_ws_bytes = (size_t)workers * (size_t)g.K * sizeof(float);
            return pl;
        }
    }
    const long long M = (long long)g.N * g.P * g.Q;
    const long long CRS = (long long)g.C * g.R * g.S;
    pl.tap = g.C >= 64;   // enough channels to fill the columns of a per-tap tile
    if (pl.tap) {
        // (bm, bn) with the least padded area, larger tile on ties
        // 96x96: three wavefronts of 96x32 each, for the 96-channel layers (fp32 kernel only)
        const int cand[9][2] = {{128, 128}, {128, 96}, {96, 128}, {192, 64}, {128, 64}, {64, 128}, {64, 64}, {32, 128}, {96, 96}};
        long long best = -1;
        for (const auto& c : cand) {
            if (c[0] == 96 && c[1] == 96 && dtype != PURINE_F32) continue;
            const long long area = (long long)((g.K + c[0] - 1) / c[0]) * c[0] * ((g.C + c[1] - 1) / c[1]) * c[1];
            if (best < 0 || area < best) { best = area; pl.bm = c[0]; pl.bn = c[1]; }
        }
        pl.c_tiles = (g.C + pl.bn - 1) / pl.bn;
        pl.tiles_j = g.R * g.S * pl.c_tiles;
    } else {
        const int cands[4] = {128, 96, 64, 32};
        long long best = -1;
        pl.bm = 32;
        for (int c : cands) {
            const long long padded = (long long)((g.K + c - 1) / c) * c;
            if (best < 0 || padded < best) { best = padded; pl.bm = c; }
        }
        pl.bn = 128;
        pl.c_tiles = 0;
        pl.tiles_j = (int)((CRS + pl.bn - 1) / pl.bn);
    }
    pl.tiles_i = (g.K + pl.bm - 1) / pl.bm;
    const long long tiles = (long long)pl.tiles_i * pl.tiles_j;
    // Number of splits. A CU holds three of these workgroups at a time, so the chip runs them in
    // rounds of 768; a grid just over a multiple of 768 leaves the chip almost idle for a whole
    // extra round, and a grid under 512 leaves too few wavefronts to hide latency. Every split also
    // writes a partial copy of dw that the second pass reads back, so more splits mean more HBM
    // traffic beside the operands. Every admissible split count gets a time estimate
    //     workgroup slots per CU x pixels per chunk x time of one tile-pixel  +  partials / bandwidth
    // and the smallest wins; chunks stay within 256..8192 pixels (a short chunk is mostly prologue
    // and epilogue, a long one lengthens the fp32 accumulation chain).
    const double rate = dtype == PURINE_F32 ? 110e12 : 450e12;      // what these kernels sustain on the MFMA units
    const double t_pixel = 2.0 * pl.bm * pl.bn * 256.0 / rate;      // one workgroup alone on a CU, per pixel
    const double dw_bytes = (double)g.K * (double)CRS * 4.0;
    const long long max_splits = (M + 255) / 256;
    long long min_splits = (M + 8191) / 8192;
    if (min_splits < 1) min_splits = 1;
    long long splits = min_splits;
    double best_time = -1.0;
    for (long long sp = min_splits; sp <= max_splits && sp <= min_splits + 4096; ++sp) {
        const long long wgs = tiles * sp;
        double slots;
        if (wgs <= 768) {
            const long long per_cu = (wgs + 255) / 256;              // 1..3 workgroups on the busiest CU
            const double hide = per_cu >= 3 ? 1.0 : (per_cu == 2 ? 0.85 : 0.55);
            slots = (double)per_cu / hide;
        } else {
            const long long rounds = (wgs + 767) / 768;
            slots = 3.0 * (double)rounds;
            // many rounds: workgroups of different rounds overlap and the tail no longer matters
            if (rounds > 6 && (double)wgs / 256.0 / 0.97 < slots) slots = (double)wgs / 256.0 / 0.97;
        }
        const double chunk_px = (double)((M + sp - 1) / sp);
        const double t = slots * chunk_px * t_pixel + 2.0 * (double)sp * dw_bytes / 4e12;
        if (best_time < 0 || t < best_time - 1e-12) { best_time = t; splits = sp; }
        if (wgs > 8 * 768) break;
    }
    long long chunk = (M + splits - 1) / splits;
    chunk = (chunk + 31) / 32 * 32;   // whole slabs of either kernel (16 or 32 pixels), 16-byte aligned rows
    splits = (M + chunk - 1) / chunk;
    pl.splits = (int)splits;
    pl.chunk = (int)chunk;
    pl.ws_bytes = (size_t)splits * (size_t)g.K * (size_t)CRS * sizeof(float);
    pl.db_ws_bytes = (size_t)splits * (size_t)g.K * sizeof(float);
    return pl;
}

hipError_t launch_conv_wgrad(int dtype, const ConvGeom& g, const WgradPlan& plan, const void* x,
                             const void* dy, float* dw, float* db, float beta, void* ws, hipStream_t st) {
    WgradParams p{};
    p.x = x; p.dy = dy;
    // bias-gradient partials [split][K] sit behind the weight-gradient partials
    p.db_out = db ? (float*)((char*)ws + wgrad_db_offset(plan)) : nullptr;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q;
    p.R = g.R; p.S = g.S; p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.PQ = g.P * g.Q; p.M = g.N * p.PQ; p.RS = g.R * g.S; p.CRS = g.C * p.RS; p.HW = g.H * g.W;
    p.div_pq = make_fastdiv(p.PQ); p.div_q = make_fastdiv(g.Q);
    p.div_rs = make_fastdiv(p.RS); p.div_s = make_fastdiv(g.S);
    p.chunk = plan.chunk; p.tiles_i = plan.tiles_i; p.tiles_j = plan.tiles_j; p.splits = plan.splits;
    p.c_tiles = plan.c_tiles;
    p.x_ns = g.x_ns; p.dy_ns = g.y_ns;
    p.out = (float*)ws;
    {
        // raw-buffer loads: two-part offsets need both tensors below 2^30 bytes
        const int es = dtype == PURINE_F32 ? 4 : 2;
        const long long xb = ((long long)(g.N - 1) * g.x_ns + (long long)g.C * p.HW) * es;
        const long long dyb = ((long long)(g.N - 1) * g.y_ns + (long long)g.K * p.PQ) * es;
        const bool ok = xb < (1LL << 30) && dyb < (1LL << 30) && !buffer_loads_disabled();
        p.x_bytes = ok ? (unsigned)xb : 0u;
        p.dy_bytes = ok ? (unsigned)dyb : 0u;
    }
    hipError_t e;
    const bool vec = p.PQ % 32 == 0 && (((uintptr_t)dy) & 15u) == 0;
    if (plan.rows) e = launch_wgrad_rows_bf16(g, plan.splits, x, dy, (float*)ws, p.db_out, st);
    else if (plan.taps) e = launch_wgrad_taps_bf16(g, x, dy, (float*)ws, p.db_out, st);
    else if (plan.cols) e = launch_wgrad_cols_bf16(g, x, dy, (float*)ws, p.db_out, st);
    else if (dtype == PURINE_F32) e = plan.tap ? dispatch_f32<true>(p, plan, st) : dispatch_f32<false>(p, plan, st);
    else if (plan.tap) e = vec ? dispatch_bf16<true, true>(p, plan, st) : dispatch_bf16<false, true>(p, plan, st);
    else e = vec ? dispatch_bf16<true, false>(p, plan, st) : dispatch_bf16<false, false>(p, plan, st);
    if (e != hipSuccess) return e;
    const int n = g.K * p.CRS;
    // 16-byte packets need aligned rows in both sets of partials (the scratch itself is aligned)
    const bool vec4 = n % 4 == 0;   // (the bias-gradient partials take an element-wise path when K % 4 != 0)
    if (vec4) {
        const int dw_blocks = (n + 31) / 32, db_blocks = db ? (g.K + 31) / 32 : 0;
        hipLaunchKernelGGL(wgrad_reduce_vec_kernel, dim3(dw_blocks + db_blocks), dim3(256), 0, st,
                           (const float*)ws, dw, n, plan.splits, beta, plan.tap ? 1 : 0, g.K, g.C, p.RS,
                           dw_blocks, (const float*)p.db_out, db);
        return hipGetLastError();
    }
    const int dw_blocks = (n + 15) / 16, db_blocks = db ? (g.K + 15) / 16 : 0;
    hipLaunchKernelGGL(wgrad_reduce_kernel, dim3(dw_blocks + db_blocks), dim3(256), 0, st,
                       (const float*)ws, dw, n, plan.splits, beta, plan.tap ? 1 : 0, g.K, g.C, p.RS,
                       dw_blocks, (const float*)p.db_out, db);
    return hipGetLastError();
}

}  // namespace purine

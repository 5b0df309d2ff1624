// bf16 MFMA variant of the pixel-major implicit GEMM (Conv / ConvBwdData, paper Figure 1(b)):
// bf16 operands, fp32 accumulation on v_mfma_f32_32x32x16_bf16, bf16 (round-to-nearest-even) output.
//
// Same contraction and the same slab walk as the fp32 tap kernel (16-byte filter pieces from the
// repacked copy, one bounds test per slab for the gathered operand), with the operand layout the
// bf16 MFMA wants: each lane feeds 8 CONSECUTIVE reduction elements of its row (A) or column (B).
// So both LDS tiles are stored reduction-major inside a row - As[i][ci], Bs[pixel][ci] - with a
// slab depth of 32 channels, and the filter is repacked to A[tap][i][ci]. NCHW keeps pixels, not
// channels, contiguous, so the gathered tensor is first copied into a channels-blocked layout
// [N][Ci_pad/8][H][W][8] in scratch (blockify_kernel, one pass at HBM speed): a thread then gathers
// 8 channels of its pixel with one 16-byte load (coalesced along W across the wavefront) and writes
// it to LDS as it is. Rows are padded to 40 elements (80 bytes) so that the 16-byte fragment reads
// of 32 rows fall in distinct bank groups. The flattened mode (fewer than 16 input channels) has
// nothing to block and gathers 2-byte elements from NCHW.
#include "pix_common.h"

namespace purine {
namespace pix {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));

constexpr int BKH = 32;        // slab depth (channels)
constexpr int LDK = BKH + 8;   // LDS row pitch in bf16 elements

// FLAT (forward with fewer than 16 input channels): the reduction is (c, r, s) flattened, Kg = Ci*R*S
// values padded to a multiple of 32, the filter copy is A[i][Kg_pad], and every gathered element
// has its own tap, walked incrementally on the scalar unit (the rows of a slab are uniform per
// wavefront) and its own bounds test, recorded as one validity bit.
// NCHW = 1 (single-tap layers, where every element is gathered exactly once and a blocked copy would
// only add traffic): tap-major walk, 2-byte gathers straight from the NCHW tensor.
// NCHW = 2: the same for layers whose gather is the identity (1x1 filter, stride 1, no padding) and
// whose planes hold an even number of pixels: a thread loads the dword that holds TWO adjacent
// pixels of a channel, and one byte-permute per output dword splits its channels' dwords into the
// two pixels' [8 channels] packets: half the load instructions and an eighth of the packing work
// of the element gather.
template <bool FLAT, int NCHW, bool MINUS, bool D2S, bool FUSED, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(WM * WN * 64) void igemm_tap_bf16_kernel(const PixParams p) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    static_assert(NT == 256 && NT % BN == 0, "whole threads per pixel column");
    constexpr int TPP = NT / BN;               // threads sharing one pixel column
    constexpr int CH = BKH / TPP;              // channels gathered per thread per slab
    static_assert(CH % 8 == 0, "16-byte LDS pieces");
    constexpr int A_CPR = BKH / 8;             // 16-byte pieces per filter row
    constexpr int A_VEC = BM * A_CPR;
    constexpr int A_ITERS = (A_VEC + NT - 1) / NT;
    constexpr int PAIRS = BN / 2;              // pixel pairs of the tile
    constexpr int TPP2 = NT / PAIRS;           // threads sharing one pixel pair
    constexpr int CH2 = BKH / TPP2;            // channels per thread per slab in the pair mode
    constexpr bool PAIR = NCHW == 2 && CH2 >= 4;   // narrower tiles keep the element gather
    constexpr bool ELEMS = FLAT || (NCHW != 0 && !PAIR);   // 2-byte gathers with per-element validity bits
    static_assert(!(FLAT && NCHW != 0), "one gather mode");

    __shared__ __attribute__((aligned(16))) uint16_t As[2][BM * LDK];
    __shared__ __attribute__((aligned(16))) uint16_t Bs[2][BN * LDK];
    __shared__ __attribute__((aligned(16))) float bias_s[FUSED ? BM : 4];   // read in 16-byte quads

    const uint16_t* __restrict__ in = (const uint16_t*)p.in;
    const uint16_t* __restrict__ wt = (const uint16_t*)p.wt;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int tile = xcd_tile(blockIdx.x, p.tiles_i * p.tiles_pix);
    const int i0 = (tile % p.tiles_i) * BM;
    const int j0 = (tile / p.tiles_i) * BN;

    // this thread's pixel column and its share of the slab's channels
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
        g_h = ho * p.g_mul_h + p.g_add_h;
        g_w = wo * p.g_mul_w + p.g_add_w;
        // FLAT: element offset in NCHW; otherwise offset in 8-channel blocks of the blocked copy
        g_off = n * (ELEMS ? p.in_ns : (p.Ci_pad / 8) * p.HiWi) + g_h * p.Wi + g_w;
    }
    const int ch_base = __builtin_amdgcn_readfirstlane(tid / BN) * CH;   // uniform per wavefront
    // pair mode: this thread's pixel pair (2*pp, 2*pp + 1 of the tile) and its CH2 channels of a slab
    int p_off = 0, p_cg = 0, p_row = 0;
    bool p_live = false, p_swap = false;
    if (PAIR) {
        const int pp = tid % PAIRS;
        p_cg = (tid / PAIRS) * CH2;
        const int pix = j0 + 2 * pp;
        p_live = pix < p.M;                    // M is even: the pair is inside or outside as a whole
        const int pc = p_live ? pix : 0;
        const int n = fastdiv(pc, p.div_howo);
        p_off = n * p.in_ns + (pc - n * p.HoWo);
        p_row = 2 * pp;
        // rows are 80 bytes: the 16 lanes of a store would hit 8 bank groups twice if all wrote their even
        // pixel; every second group of 8 lanes writes its odd pixel first
        p_swap = (pp >> 3) & 1;
    }
    // the blocked copy as a raw buffer (not used by the 2-byte gather modes)
    const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>(in), (short)0, ELEMS ? 0 : (int)p.in_bytes, 0x00020000);

    int a_src[A_ITERS], a_dst[A_ITERS];
#pragma unroll
    for (int it = 0; it < A_ITERS; ++it) {
        const int f = tid + it * NT;
        const int row = f / A_CPR, piece = f - row * A_CPR;
        a_src[it] = (f < A_VEC) ? (i0 + row) * p.Ci_pad + piece * 8 : -1;
        a_dst[it] = row * LDK + piece * 8;
    }

    typedef unsigned u32x4_t __attribute__((ext_vector_type(4)));   // native vector: stays in registers
    u32x4_t a_reg[A_ITERS];
    uint32_t b_reg[ELEMS ? CH : 1];  // FLAT / NCHW: raw 16-bit values
    uint32_t pr_reg[PAIR ? CH2 : 1]; // pair mode: one dword (two pixels) per channel
    uint4 blk_reg[CH / 8];           // blocked input: 8 channels of this thread's pixel per piece
    bool b_ok = false;
    uint32_t b_bits = 0;             // FLAT / NCHW: validity of each gathered element

    int nx_r = 0, nx_s = 0, nx_c0 = 0;
    auto load_slab = [&]() {
        const int tap = FLAT ? 0 : nx_r * p.St + nx_s;
        const int a_slab = tap * p.i_pad * p.Ci_pad + nx_c0;
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it)
            if (a_src[it] >= 0) a_reg[it] = *reinterpret_cast<const u32x4_t*>(wt + a_slab + a_src[it]);
        if (FLAT) {
            // this wavefront's run of CH flattened rows starts at kk0 = (c, r, s)
            int kk = nx_c0 + ch_base;
            const int kq = kk < p.Kg ? kk : 0;
            int w_c = fastdiv(kq, p.div_rs);
            const int rs = kq - w_c * p.RS;
            int w_r = fastdiv(rs, p.div_s);
            int w_s = rs - w_r * p.S;
            int w_off = w_c * p.HiWi + w_r * p.Wi + w_s;
            b_bits = 0;
#pragma unroll
            for (int e = 0; e < CH; ++e) {
                const int hi = g_h + w_r, wi = g_w + w_s;
                // bitwise & on purpose: no short-circuit control flow inside the slab loop
                const bool ok = g_live & (kk < p.Kg) & ((unsigned)hi < (unsigned)p.Hi) & ((unsigned)wi < (unsigned)p.Wi);
                b_reg[ELEMS ? e : 0] = in[ok ? g_off + w_off : 0];     // clamped: masked at the store
                b_bits |= (ok ? 1u : 0u) << e;
                // next row, branch-free (selects on the scalar unit)
                kk += 1; w_s += 1;
                const bool wrap_s = w_s >= p.S;
                w_s = wrap_s ? 0 : w_s;
                w_r += wrap_s ? 1 : 0;
                const bool wrap_r = w_r >= p.R;
                w_r = wrap_r ? 0 : w_r;
                w_off += 1 + (wrap_s ? p.Wi - p.S : 0) + (wrap_r ? p.HiWi - p.R * p.Wi : 0);
            }
            nx_c0 += BKH;
            nx_c0 = nx_c0 >= p.Ci_pad ? 0 : nx_c0;
            return;
        }
        if (PAIR) {
            b_bits = 0;
#pragma unroll
            for (int e = 0; e < (PAIR ? CH2 : 0); ++e) {
                const int ci = nx_c0 + p_cg + e;
                const bool ok = p_live & (ci < p.Ci);
                pr_reg[PAIR ? e : 0] = *reinterpret_cast<const uint32_t*>(in + (ok ? p_off + ci * p.HiWi : 0));   // clamped: masked at the store
                b_bits |= (ok ? 1u : 0u) << e;
            }
            nx_c0 += BKH;
            nx_c0 = nx_c0 >= p.Ci_pad ? 0 : nx_c0;
            return;
        }
        const int hi = MINUS ? g_h - nx_r : g_h + nx_r;
        const int wi = MINUS ? g_w - nx_s : g_w + nx_s;
        const int tap_off = nx_r * p.Wi + nx_s;
        b_ok = g_live & ((unsigned)hi < (unsigned)p.Hi) & ((unsigned)wi < (unsigned)p.Wi);
        const int base = MINUS ? g_off - tap_off : g_off + tap_off;
        if (NCHW != 0) {
            b_bits = 0;
#pragma unroll
            for (int e = 0; e < CH; ++e) {
                const int ci = nx_c0 + ch_base + e;
                const bool ok = b_ok & (ci < p.Ci);
                b_reg[ELEMS ? e : 0] = in[ok ? base + ci * p.HiWi : 0];   // clamped: masked at the store
                b_bits |= (ok ? 1u : 0u) << e;
            }
        }
        // blocked copy, read as a raw buffer: a masked lane carries byte offset 2^31, which the
        // hardware range check answers with zeros (the copy is below 2^31 bytes, checked on the host)
        const unsigned vbase = b_ok ? (unsigned)base * 16u : 0x80000000u;
#pragma unroll
        for (int q = 0; q < (NCHW != 0 ? 0 : CH / 8); ++q) {
            const int cb = ((nx_c0 + ch_base) >> 3) + q;                 // zero blocks pad Ci to Ci_pad
            typedef unsigned u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsrc, vbase, cb * p.HiWi * 16, 0);
            blk_reg[q] = make_uint4(v[0], v[1], v[2], v[3]);
        }
        // all taps of one channel group back to back (halo rows stay in L1/L2), then the next group
        nx_s += 1;
        const bool wrap_s = nx_s >= p.St;
        nx_s = wrap_s ? 0 : nx_s;
        nx_r += wrap_s ? 1 : 0;
        const bool wrap_r = nx_r >= p.Rt;
        nx_r = wrap_r ? 0 : nx_r;
        nx_c0 += wrap_r ? BKH : 0;
        nx_c0 = nx_c0 >= p.Ci_pad ? 0 : nx_c0;
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it)
            if (a_src[it] >= 0) *reinterpret_cast<u32x4_t*>(&As[buf][a_dst[it]]) = a_reg[it];
        if (PAIR) {
            uint32_t ev[CH2 / 2], od[CH2 / 2];   // channel pairs of the even and of the odd pixel
#pragma unroll
            for (int h = 0; h < CH2 / 2; ++h) {
                const uint32_t c0 = ((b_bits >> (2 * h)) & 1u) ? pr_reg[PAIR ? 2 * h : 0] : 0u;
                const uint32_t c1 = ((b_bits >> (2 * h + 1)) & 1u) ? pr_reg[PAIR ? 2 * h + 1 : 0] : 0u;
                ev[h] = __builtin_amdgcn_perm(c1, c0, 0x05040100u);
                od[h] = __builtin_amdgcn_perm(c1, c0, 0x07060302u);
            }
            uint16_t* first = &Bs[buf][(p_row + (p_swap ? 1 : 0)) * LDK + p_cg];
            uint16_t* second = &Bs[buf][(p_row + (p_swap ? 0 : 1)) * LDK + p_cg];
#pragma unroll
            for (int q = 0; q < CH2 / 4; ++q) {   // 8-byte pieces (4 channels)
                const uint2 f = make_uint2(p_swap ? od[2 * q] : ev[2 * q], p_swap ? od[2 * q + 1] : ev[2 * q + 1]);
                const uint2 g = make_uint2(p_swap ? ev[2 * q] : od[2 * q], p_swap ? ev[2 * q + 1] : od[2 * q + 1]);
                *reinterpret_cast<uint2*>(first + q * 4) = f;
                *reinterpret_cast<uint2*>(second + q * 4) = g;
            }
            return;
        }
        uint16_t* row = &Bs[buf][(tid % BN) * LDK + ch_base];
        if (!ELEMS) {
#pragma unroll
            for (int q = 0; q < CH / 8; ++q)
                *reinterpret_cast<uint4*>(row + q * 8) = blk_reg[q];   // zeros came from the loads
            return;
        }
#pragma unroll
        for (int q = 0; q < CH / 8; ++q) {
            uint32_t w[4];
#pragma unroll
            for (int h = 0; h < 4; ++h) {
                const int e = q * 8 + 2 * h;
                const uint32_t lo = ((b_bits >> e) & 1u) ? b_reg[ELEMS ? e : 0] : 0u;
                const uint32_t hi = ((b_bits >> (e + 1)) & 1u) ? b_reg[ELEMS ? e + 1 : 0] : 0u;
                w[h] = lo | (hi << 16);
            }
            *reinterpret_cast<uint4*>(row + q * 8) = make_uint4(w[0], w[1], w[2], w[3]);
        }
    };

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

    const int n_slabs = (FLAT ? 1 : p.Rt * p.St) * (p.Ci_pad / BKH);
    load_slab();
    if (FUSED) stage_bias<uint16_t, BM, NT>(bias_s, p, i0, tid);
    store_slab(0);
    __syncthreads();

    const int a_row = (wm * TM * 32 + (lane & 31)) * LDK + (lane >> 5) * 8;
    const int b_row = (wn * TN * 32 + (lane & 31)) * LDK + (lane >> 5) * 8;

    for (int slab = 0; slab < n_slabs; ++slab) {
        const int buf = slab & 1;
        load_slab();
#pragma unroll
        for (int ks = 0; ks < BKH / 16; ++ks) {
            bf16x8 av[TM], bv[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a)
                av[a] = *reinterpret_cast<const bf16x8*>(&As[buf][a_row + a * 32 * LDK + ks * 16]);
#pragma unroll
            for (int b = 0; b < TN; ++b)
                bv[b] = *reinterpret_cast<const bf16x8*>(&Bs[buf][b_row + b * 32 * LDK + ks * 16]);
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[a], bv[b], acc[a][b], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        store_slab(buf ^ 1);
        __syncthreads();
    }

    store_tile<uint16_t, D2S, FUSED, TM, TN, !MINUS>(p, (uint16_t*)p.out, acc, i0 + wm * TM * 32,
                                      j0 + wn * TN * 32 + (lane & 31), lane >> 5, bias_s, i0);
}

// NCHW -> [N][CBp][HW][8]: thread = (image, channel block, pixel); channels past C are zero.
__global__ __launch_bounds__(256) void blockify_kernel(const uint16_t* __restrict__ src, uint4* __restrict__ dst,
                                                       int C, int HW, int CBp, long long total, long long src_ns) {
    for (long long o = (long long)blockIdx.x * 256 + threadIdx.x; o < total; o += (long long)gridDim.x * 256) {
        const long long plane = o / HW;                  // n * CBp + cb
        const int pix = (int)(o - plane * HW);
        const int cb = (int)(plane % CBp);
        const long long n = plane / CBp;
        const uint16_t* s = src + n * src_ns + (long long)cb * 8 * HW + pix;
        uint32_t v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = cb * 8 + e < C ? (uint32_t)s[(long long)e * HW] : 0u;
        dst[o] = make_uint4(v[0] | (v[1] << 16), v[2] | (v[3] << 16), v[4] | (v[5] << 16), v[6] | (v[7] << 16));
    }
}

template <bool FLAT, int NCHW, bool MINUS, bool D2S, bool FUSED, int TM, int TN, int WM, int WN>
hipError_t launch_one(PixParams& p, hipStream_t st) {
    const long long total = (long long)p.tiles_i * p.tiles_pix;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    hipLaunchKernelGGL((igemm_tap_bf16_kernel<FLAT, NCHW, MINUS, D2S, FUSED, TM, TN, WM, WN>), dim3((unsigned)total),
                       dim3(WM * WN * 64), 0, st, p);
    return hipGetLastError();
}

template <bool FLAT, int NCHW, bool MINUS, bool D2S, bool FUSED>
hipError_t by_tile2(PixParams& p, int bm, int bn, hipStream_t st) {
#define CALL(TM, TN, WM, WN) launch_one<FLAT, NCHW, MINUS, D2S, FUSED, TM, TN, WM, WN>(p, st)
    PURINE_TILE_SWITCH(CALL)
#undef CALL
}
template <bool FLAT, int NCHW, bool MINUS, bool D2S>
hipError_t by_tile(PixParams& p, int bm, int bn, hipStream_t st) {
    const bool fused = p.bias || p.relu || p.mask;
    return fused ? by_tile2<FLAT, NCHW, MINUS, D2S, true>(p, bm, bn, st)
                 : by_tile2<FLAT, NCHW, MINUS, D2S, false>(p, bm, bn, st);
}

}  // namespace

// Channels-blocked copy of the gathered tensor (p.in, [N][Ci][Hi][Wi] bf16) into `blocked`
// ([N][Ci_pad/8][Hi][Wi][8]); p.in is redirected to it.
hipError_t blockify_input(PixParams& p, void* blocked, hipStream_t st) {
    const int CBp = p.Ci_pad / 8;
    const long long total = (long long)p.N * CBp * p.HiWi;
    // the kernels address the copy with byte offsets below 2^31
    if (total <= 0 || total * 16 >= 0x7fffffffLL) return hipErrorInvalidValue;
    p.in_bytes = (unsigned)(total * 16);
    const long long blocks = (total + 255) / 256;
    (void)hipGetLastError();
    hipLaunchKernelGGL(blockify_kernel, dim3((unsigned)(blocks > 1048576 ? 1048576 : blocks)), dim3(256), 0, st,
                       (const uint16_t*)p.in, (uint4*)blocked, p.Ci, p.HiWi, CBp, total, (long long)p.in_ns);
    p.in = blocked;
    return hipGetLastError();
}

hipError_t dispatch_tap_bf16(PixParams& p, int mode, int bm, int bn, hipStream_t st) {
    if (mode == 0) return by_tile<false, 0, false, false>(p, bm, bn, st);
    if (mode == 1) return by_tile<false, 0, true, false>(p, bm, bn, st);
    return by_tile<false, 0, true, true>(p, bm, bn, st);
}

// single-tap layers: gathers from the NCHW tensor p.in itself. A strided backward-data pass whose
// filter fits inside one stride step (R <= sh, S <= sw) is phase-folded onto a single tap too, and
// needs the depth-to-space epilogue like any other phase-folded pass.
hipError_t dispatch_tap_bf16_nchw(PixParams& p, int mode, int bm, int bn, hipStream_t st) {
    // identity gather with whole pixel pairs: the pair mode
    const bool identity = p.Rt == 1 && p.St == 1 && p.g_mul_h == 1 && p.g_mul_w == 1 && p.g_add_h == 0 && p.g_add_w == 0 &&
                          p.Hi == p.Ho && p.Wi == p.Wo;
    if (identity && mode != 2 && ((p.HoWo | p.in_ns) & 1) == 0 && (((uintptr_t)p.in) & 3u) == 0) {
        if (mode == 0) return by_tile<false, 2, false, false>(p, bm, bn, st);
        return by_tile<false, 2, true, false>(p, bm, bn, st);
    }
    if (mode == 0) return by_tile<false, 1, false, false>(p, bm, bn, st);
    if (mode == 1) return by_tile<false, 1, true, false>(p, bm, bn, st);
    return by_tile<false, 1, true, true>(p, bm, bn, st);
}

// forward, flattened (c, r, s) reduction; p.wt is the filter copy A[i_pad][Ci_pad] with Ci_pad = Kg
// rounded up to a multiple of 32, p.Rt = p.St = 1
hipError_t dispatch_flat_bf16(PixParams& p, int bm, int bn, hipStream_t st) {
    return by_tile<true, 0, false, false>(p, bm, bn, st);
}

}  // namespace pix
}  // namespace purine

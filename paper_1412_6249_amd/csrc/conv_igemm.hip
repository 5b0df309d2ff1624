// Pixel-major implicit-GEMM convolution for gfx950: the Conv and ConvBwdData operators of the
// convolution layer (paper Figure 1(b)).
//
// Both passes are the contraction
//     out[n, i, ho, wo] = sum over taps (r, s) and gathered channels ci of
//                         A[(r,s), ci, i] * in[n, ci, h(ho, r), w(wo, s)]
// i.e. a GEMM whose B operand is the patch matrix of the gathered tensor. That matrix is never
// stored in HBM: each workgroup builds a 16 x BN slab of it in LDS straight from the NCHW tensor
// (lanes run along pixels, so loads are coalesced along W), multiplies it with a 16 x BM slab of
// the filter matrix on the fp32 MFMA units and keeps the BM x BN output tile in accumulators.
//
//   forward                 : in = x,  i = k,       ci = c, h = ho*sh - ph + r
//   backward-data, stride 1 : in = dy, i = c,       ci = k, h = ho + ph - r
//   backward-data, strided  : in = dy, i = (c,a,b), ci = k, h = hq - r'   (phase-folded, below)
//
// A slab of the reduction is 16 consecutive channels ci of ONE tap (r, s). Within a slab the bounds
// test and the tap offset are the same for all 16 rows, so a gathered element costs one add and
// one load; the slabs of one channel group walk through all its taps before the next group, so the
// halo rows the taps share stay in L1/L2. The filter is first repacked (a tiny kernel, into caller
// scratch) to A[(r,s)][ci][i], zero padded to whole slabs and tiles, which makes the filter slab a
// dense block read with unconditional 16-byte loads. Layers with fewer than 16 gathered channels (the
// first layer of a CNN, forward) would waste most of a slab, so they run a second kernel that
// flattens (c, r, s) into one reduction index instead.
//
// MFMA operand roles: A rows = channels i, B columns = pixels, so each accumulator register holds
// 32 consecutive pixels of one channel and the NCHW stores are 128-byte coalesced.
#include "pix_common.h"

namespace purine {
namespace {

using namespace pix;

constexpr int BK = 16;  // slab depth along the reduction (fp32 kernels)

// ------------------------------------------------------------------------------------------------
// Tap-major kernel. MINUS: the gather walks backwards (h = g_h - r), as backward-data does.
// D2S: depth-to-space epilogue of the phase-folded strided backward-data.
// Workgroup = WM x WN wavefronts, each owning TM x TN MFMA tiles of MT x MT: 32 (v_mfma 32x32x2) or
// 16 (v_mfma 16x16x4, same flop rate, for GEMMs whose row count would waste half a 32-row tile).
// BUF: the gathered operand is read with raw buffer loads. The hardware range check (byte offset =
// per-lane part + scalar part against the tensor's size) returns zero for an out-of-range offset,
// so a masked lane carries offset 2^31 and a padding channel a scalar offset of 2^31 - 1, and the
// slab loop needs neither the clamped addresses nor the zero-fill selects. The host enables it for
// tensors below 2^31 bytes.
template <typename T, bool MINUS, bool D2S, bool FUSED, int TM, int TN, int WM, int WN, int MT = 32, bool BUF = false>
__global__ __launch_bounds__(WM * WN * 64, (MT == 32 && TM == 2 && TN == 2 && WM == 2 ? 4 : (MT == 16 && TM == 3 && TN == 2 && BUF ? 7 : 1)))
void igemm_tap_kernel(const PixParams p) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * MT;
    constexpr int BN = WN * TN * MT;
    constexpr int KSTEP = MT == 32 ? 2 : 4;    // reduction elements per MFMA
    // 16-wide tiles: a fragment read takes four consecutive slab rows at once (16 lanes each), so odd
    // rows are stored with bit 4 of the column flipped: rows r and r+1 then sit 16 banks apart without
    // padding, and the 48x128 tile's 22.5 KB let seven workgroups share a CU's LDS.
    constexpr int LDB = BN;
    constexpr int SWZ = MT == 16 ? 16 : 0;
    static_assert(MT == 32 || MT == 16, "MFMA tile edge");
    static_assert(NT == 256 && NT % BN == 0, "one pixel column per thread");
    constexpr int B_RPP = NT / BN;             // slab rows covered per pass
    constexpr int B_PASSES = BK / B_RPP;
    constexpr int A_VEC = BK * BM / 4;         // 16-byte pieces of the filter slab
    constexpr int A_ITERS = (A_VEC + NT - 1) / NT;
    constexpr int A_CPR = BM / 4;              // pieces per slab row

    __shared__ __attribute__((aligned(16))) float As[2][BK * BM];
    __shared__ float Bs[2][BK * LDB];
    __shared__ __attribute__((aligned(16))) float bias_s[FUSED ? BM : 4];   // read in 16-byte quads

    const T* __restrict__ in = (const T*)p.in;
    const T* __restrict__ wt = (const T*)p.wt;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int tile = xcd_tile(blockIdx.x, p.tiles_i * p.tiles_pix);
    const int i0 = (tile % p.tiles_i) * BM;
    const int j0 = (tile / p.tiles_i) * BN;

    // ---- this thread's pixel column of the patch slab (fixed for the whole kernel) ----
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
        g_off = n * p.in_ns + g_h * p.Wi + g_w;   // tap (0,0) of channel 0
    }
    const int b_row = __builtin_amdgcn_readfirstlane(tid / BN);  // uniform per wavefront (BN >= 64)
    // descriptor of the gathered tensor as a raw buffer of p.in_bytes bytes (BUF only)
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(in), (short)0, BUF ? (int)p.in_bytes : 0, 0x00020000);

    // filter slab pieces served by this thread: element offset inside a slab, and LDS slot
    int a_src[A_ITERS], a_dst[A_ITERS];
#pragma unroll
    for (int it = 0; it < A_ITERS; ++it) {
        const int f = tid + it * NT;
        const int row = f / A_CPR, col = (f - row * A_CPR) * 4;
        a_src[it] = (f < A_VEC) ? row * p.i_pad + i0 + col : -1;
        a_dst[it] = row * BM + col;
    }

    floatx4 a_reg[A_ITERS];
    float b_reg[B_PASSES];
    bool b_ok;

    // Scalar walk over the slabs: tap (nx_r, nx_s) and first channel nx_c0 of the next slab to load.
    // Taps are the INNER loop: all taps of one 16-channel group are visited back to back, so the
    // halo rows they share are re-read while still in L1/L2 (walking the channels inside a tap
    // re-fetched the gathered tensor from beyond L2 once per tap).
    int nx_r = 0, nx_s = 0, nx_c0 = 0, staged_c0 = 0;
    auto load_slab = [&]() {
        staged_c0 = nx_c0;
        const int tap = nx_r * p.St + nx_s;
        const int a_slab = (tap * p.Ci_pad + nx_c0) * p.i_pad;
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it)
            if (a_src[it] >= 0) a_reg[it] = Elem<T>::load4(wt, a_slab + a_src[it]);
        const int hi = MINUS ? g_h - nx_r : g_h + nx_r;
        const int wi = MINUS ? g_w - nx_s : g_w + nx_s;
        const int tap_off = nx_r * p.Wi + nx_s;
        b_ok = g_live & ((unsigned)hi < (unsigned)p.Hi) & ((unsigned)wi < (unsigned)p.Wi);
        if (BUF) {
            const unsigned vbase = b_ok ? (unsigned)(MINUS ? g_off - tap_off : g_off + tap_off) * 4u : 0x80000000u;
#pragma unroll
            for (int ps = 0; ps < B_PASSES; ++ps) {
                const int ci = nx_c0 + ps * B_RPP + b_row;                   // uniform per wavefront
                const int soff = ci < p.Ci ? ci * p.HiWi * 4 : 0x7fffffff;   // scalar part of the offset
                b_reg[ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, vbase, soff, 0));
            }
        } else {
            const int base = b_ok ? (MINUS ? g_off - tap_off : g_off + tap_off) : 0;
#pragma unroll
            for (int ps = 0; ps < B_PASSES; ++ps) {
                const int ci = nx_c0 + ps * B_RPP + b_row;
                // rows past Ci (padding of the last slab of a tap) read channel 0 and are zeroed at the store
                const int plane = (b_ok & (ci < p.Ci)) ? ci * p.HiWi : 0;
                b_reg[ps] = Elem<T>::load(in, base + plane);
            }
        }
        // advance to the next slab (past the last one it wraps to the start; those values are unused)
        nx_s += 1;
        const bool wrap_s = nx_s >= p.St;
        nx_s = wrap_s ? 0 : nx_s;
        nx_r += wrap_s ? 1 : 0;
        const bool wrap_r = nx_r >= p.Rt;
        nx_r = wrap_r ? 0 : nx_r;
        nx_c0 += wrap_r ? BK : 0;
        nx_c0 = nx_c0 >= p.Ci_pad ? 0 : nx_c0;
    };
    auto store_slab = [&](int buf) {
        const int c0 = staged_c0;
#pragma unroll
        for (int it = 0; it < A_ITERS; ++it)
            if (a_src[it] >= 0) *reinterpret_cast<floatx4*>(&As[buf][a_dst[it]]) = a_reg[it];
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps) {
            const bool ok = BUF | (b_ok & (c0 + ps * B_RPP + b_row < p.Ci));   // BUF: zeros came from the loads
            const int row = ps * B_RPP + b_row;
            Bs[buf][row * LDB + ((tid % BN) ^ ((row & 1) * SWZ))] = ok ? b_reg[ps] : 0.0f;
        }
    };

    typedef typename AccT<MT>::type acc_t;
    acc_t acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < AccT<MT>::N; ++e) acc[a][b][e] = 0.0f;

    const int n_slabs = p.Rt * p.St * (p.Ci_pad / BK);
    load_slab();
    if (FUSED) stage_bias<T, BM, NT>(bias_s, p, i0, tid);
    store_slab(0);
    __syncthreads();

    const int a_off = wm * TM * MT + (lane & (MT - 1));
    const int b_off = wn * TN * MT + (lane & (MT - 1));
    const int khalf = lane / MT;      // which of the KSTEP reduction elements this lane feeds
    int b_col[TN];                    // this lane's column of each of its MFMA tiles (KSTEP is even: row parity = khalf's)
#pragma unroll
    for (int b = 0; b < TN; ++b) b_col[b] = (b_off + b * MT) ^ ((khalf & 1) * SWZ);

    for (int slab = 0; slab < n_slabs; ++slab) {
        const int buf = slab & 1;
        load_slab();   // global loads of the next slab fly while the MFMAs below run
        float av[2][TM], bv[2][TN];   // operand fragments, double-buffered across k-steps
#pragma unroll
        for (int a = 0; a < TM; ++a) av[0][a] = As[buf][khalf * BM + a_off + a * MT];
#pragma unroll
        for (int b = 0; b < TN; ++b) bv[0][b] = Bs[buf][khalf * LDB + b_col[b]];
#pragma unroll
        for (int ks = 0; ks < BK / KSTEP; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks + 1 < BK / KSTEP) {
                const int row = KSTEP * (ks + 1) + khalf;
#pragma unroll
                for (int a = 0; a < TM; ++a) av[nxt][a] = As[buf][row * BM + a_off + a * MT];
#pragma unroll
                for (int b = 0; b < TN; ++b) bv[nxt][b] = Bs[buf][row * LDB + b_col[b]];
            }
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = AccT<MT>::mfma(av[cur][a], bv[cur][b], acc[a][b]);
        }
        __builtin_amdgcn_sched_barrier(0);   // keep the LDS stores (and their load waits) below the MFMAs
        store_slab(buf ^ 1);
        __syncthreads();
    }

    store_tile<T, D2S, FUSED, TM, TN, !MINUS>(p, (T*)p.out, acc, i0 + wm * TM * MT, j0 + b_off, khalf, bias_s, i0);
}

// ------------------------------------------------------------------------------------------------
// Flat kernel: forward pass of layers with fewer than 16 input channels. The reduction index is
// kk = (c, r, s) flattened, which equals the memory order of one filter row; the offset and tap of
// every row are decoded once per workgroup into an LDS table.
// BUF: raw buffer loads as in the tap kernel; a row past the end of the reduction carries byte offset
// 2^30 in the table and a pixel that does not exist 2^31, so (tensor below 2^30 bytes) their sums
// are out of range and read as zero.
template <typename T, bool FUSED, bool NOPAD, bool BUF, int TM, int TN, int WM, int WN>
// 96x256 tile: three workgroups per CU fit the LDS; the bound keeps the fused variant's registers
// (whose epilogue would otherwise copy all 96 accumulators out at once) within that occupancy too.
__global__ __launch_bounds__(WM * WN * 64, (TM * TN == 6 && BUF && NOPAD ? 3 : 1)) void igemm_flat_kernel(const PixParams p) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    constexpr int LDA = BM + 2;   // +2: the transposed filter-slab store hits distinct banks
    static_assert(NT == 256 && NT % BN == 0, "one pixel column per thread");
    constexpr int B_RPP = NT / BN;
    constexpr int B_PASSES = BK / B_RPP;
    constexpr int A_RPP = NT / BK;
    constexpr int A_PASSES = BM / A_RPP;
    static_assert(BM % A_RPP == 0, "filter mapping");

    __shared__ float As[2][BK * LDA];
    __shared__ float Bs[2][BK * BN];
    __shared__ __attribute__((aligned(16))) float bias_s[FUSED ? BM : 4];   // read in 16-byte quads
    __shared__ int tab_off[FLAT_MAX_KG];
    __shared__ int tab_rs[NOPAD ? 1 : FLAT_MAX_KG];

    const T* __restrict__ in = (const T*)p.in;
    const T* __restrict__ wt = (const T*)p.wt;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int tile = xcd_tile(blockIdx.x, p.tiles_i * p.tiles_pix);
    const int i0 = (tile % p.tiles_i) * BM;
    const int j0 = (tile / p.tiles_i) * BN;

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
        g_off = n * p.in_ns + g_h * p.Wi + g_w;
    }
    const int b_row = __builtin_amdgcn_readfirstlane(tid / BN);
    const int a_kk = tid % BK;
    const int a_i = tid / BK;

    float a_reg[A_PASSES];
    float b_reg[B_PASSES];
    unsigned a_ok, b_ok;   // one validity bit per staged value; the zero-fill happens at the LDS store

    // Row kk = (c, r, s) of the flattened reduction: offset c*Hi*Wi + r*Wi + s inside one image and
    // its tap, decoded once per workgroup into LDS (the host guarantees Kg <= FLAT_MAX_KG); a
    // wavefront's rows are uniform across its lanes, so the lookups are broadcast reads.
    const int n_rows = (p.Kg + BK - 1) / BK * BK;
    for (int k = tid; k < n_rows; k += NT) {
        const int kq = k < p.Kg ? k : 0;
        const int c = fastdiv(kq, p.div_rs);
        const int rs = kq - c * p.RS;
        const int r = fastdiv(rs, p.div_s);
        const int sx = rs - r * p.S;
        tab_off[k] = BUF ? (k < p.Kg ? (c * p.HiWi + r * p.Wi + sx) * 4 : 0x40000000) : c * p.HiWi + r * p.Wi + sx;
        if (!NOPAD) tab_rs[k] = (r << 16) | sx;
    }
    __syncthreads();
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(in), (short)0, BUF ? (int)p.in_bytes : 0, 0x00020000);
    const unsigned g_voff = g_live ? (unsigned)g_off * 4u : 0x80000000u;
    // BUF: the filter [Co][Kg] is read the same way: a per-row byte offset fixed for the kernel
    // (marker 2^30 for a row past Co) plus a per-slab column offset (marker 2^31 past Kg; without it
    // the column would run on into the next row). The host enables BUF only for filters below 2^30 bytes.
    const __amdgpu_buffer_rsrc_t rs_w =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<T*>(wt), (short)0, BUF ? p.Co * p.Kg * 4 : 0, 0x00020000);
    unsigned a_voff[BUF ? A_PASSES : 1];
    if (BUF) {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps) {
            const int i = i0 + a_i + ps * A_RPP;
            a_voff[BUF ? ps : 0] = i < p.Co ? (unsigned)(i * p.Kg) * 4u : 0x40000000u;
        }
    }

    auto load_slab = [&](int slab) {
        a_ok = 0u; b_ok = 0u;
        {
            const int kk = slab * BK + a_kk;
            const bool kv = kk < p.Kg;
            if (BUF) {
                const unsigned a_k = kv ? (unsigned)kk * 4u : 0x80000000u;
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps)
                    a_reg[ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rs_w, a_k + a_voff[BUF ? ps : 0], 0, 0));
            } else {
#pragma unroll
                for (int ps = 0; ps < A_PASSES; ++ps) {
                    const int i = i0 + a_i + ps * A_RPP;
                    const bool ok = kv & (i < p.Co);
                    a_reg[ps] = Elem<T>::load(wt, ok ? i * p.Kg + kk : 0);   // clamped, branch-free
                    a_ok |= (ok ? 1u : 0u) << ps;
                }
            }
        }
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps) {
            const int kk = slab * BK + ps * B_RPP + b_row;       // uniform per wavefront
            const int kc = kk < n_rows ? kk : 0;                 // the slab past the end is all masked
            bool ok = (kk < p.Kg) & g_live;
            if (!NOPAD) {
                const int rs = tab_rs[kc];
                const int hi = g_h + (rs >> 16), wi = g_w + (rs & 0xffff);
                // bitwise & on purpose: no short-circuit control flow inside the slab loop
                ok = ok & ((unsigned)hi < (unsigned)p.Hi) & ((unsigned)wi < (unsigned)p.Wi);
            }
            if (BUF) {
                const unsigned v = g_voff + (unsigned)tab_off[kc];
                b_reg[ps] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, (NOPAD || ok) ? v : 0x80000000u, 0, 0));
            } else {
                b_reg[ps] = Elem<T>::load(in, ok ? g_off + tab_off[kc] : 0);
                b_ok |= (ok ? 1u : 0u) << ps;
            }
        }
    };
    auto store_slab = [&](int buf) {
#pragma unroll
        for (int ps = 0; ps < A_PASSES; ++ps)
            As[buf][a_kk * LDA + a_i + ps * A_RPP] = (BUF || ((a_ok >> ps) & 1u)) ? a_reg[ps] : 0.0f;
#pragma unroll
        for (int ps = 0; ps < B_PASSES; ++ps)
            Bs[buf][(ps * B_RPP + b_row) * BN + (tid % BN)] = (BUF || ((b_ok >> ps) & 1u)) ? b_reg[ps] : 0.0f;
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
    if (FUSED) stage_bias<T, BM, NT>(bias_s, p, i0, tid);
    store_slab(0);
    __syncthreads();

    const int a_off = wm * TM * 32 + (lane & 31);
    const int b_off = wn * TN * 32 + (lane & 31);
    const int khalf = lane >> 5;

    for (int slab = 0; slab < n_slabs; ++slab) {
        const int buf = slab & 1;
        load_slab(slab + 1);   // past the end: every value is masked to zero
        float av[2][TM], bv[2][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a) av[0][a] = As[buf][khalf * LDA + a_off + a * 32];
#pragma unroll
        for (int b = 0; b < TN; ++b) bv[0][b] = Bs[buf][khalf * BN + b_off + b * 32];
#pragma unroll
        for (int ks = 0; ks < BK / 2; ++ks) {
            const int cur = ks & 1, nxt = cur ^ 1;
            if (ks + 1 < BK / 2) {
                const int row = 2 * (ks + 1) + khalf;
#pragma unroll
                for (int a = 0; a < TM; ++a) av[nxt][a] = As[buf][row * LDA + a_off + a * 32];
#pragma unroll
                for (int b = 0; b < TN; ++b) bv[nxt][b] = Bs[buf][row * BN + b_off + b * 32];
            }
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[cur][a], bv[cur][b], acc[a][b], 0, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        store_slab(buf ^ 1);
        __syncthreads();
    }

    store_tile<T, false, FUSED, TM, TN, true>(p, (T*)p.out, acc, i0 + wm * TM * 32, j0 + b_off, khalf, bias_s, i0);
}

// ------------------------------------------------------------------------------------------------
// Filter repack: A[tap][ci][i] (or A[tap][i][ci] for the bf16 MFMA kernel) with zero padding, from
// the KCRS filter.
//   mode 0 (forward)        : tap = (r, s),   ci = c, i = k
//   mode 1 (bwd, stride 1)  : tap = (r, s),   ci = k, i = c
//   mode 2 (bwd, strided)   : tap = (r', s'), ci = k, i = (c, a, b) -> w[k, c, a + sh*r', b + sw*s']
//   mode 3 (fwd, flattened) : one tap, ci = (c, r, s) flattened (Ci = C*R*S), i = k
struct RepackParams {
    const void* w; void* a;
    int mode, K, C, R, S, sh, sw, St, Ci, Co, Ci_pad, i_pad, total;
    int i_major;   // 0: A[tap][ci][i] (fp32 kernels), 1: A[tap][i][ci] (bf16 MFMA kernel)
};

template <typename T>
__global__ __launch_bounds__(256) void repack_filter_kernel(const RepackParams q) {
    const T* __restrict__ w = (const T*)q.w;
    T* __restrict__ a = (T*)q.a;
    for (int o = blockIdx.x * 256 + threadIdx.x; o < q.total; o += gridDim.x * 256) {
        int i, ci, tap;
        if (q.i_major) {
            ci = o % q.Ci_pad;
            const int t = o / q.Ci_pad;
            i = t % q.i_pad;
            tap = t / q.i_pad;
        } else {
            i = o % q.i_pad;
            const int t = o / q.i_pad;
            ci = t % q.Ci_pad;
            tap = t / q.Ci_pad;
        }
        const int tr = tap / q.St, ts = tap - tr * q.St;
        T v = (T)0;
        if (i < q.Co && ci < q.Ci) {
            int k, c, r, s;
            if (q.mode == 3) { a[o] = w[i * q.Ci + ci]; continue; }   // flattened: ci runs over (c, r, s)
            if (q.mode == 0) { k = i; c = ci; r = tr; s = ts; }
            else if (q.mode == 1) { k = ci; c = i; r = tr; s = ts; }
            else {
                const int ph = q.sh * q.sw;
                c = i / ph;
                const int ab = i - c * ph;
                const int pa = ab / q.sw, pb = ab - pa * q.sw;
                k = ci; r = pa + q.sh * tr; s = pb + q.sw * ts;
            }
            if (r < q.R && s < q.S) v = w[((k * q.C + c) * q.R + r) * q.S + s];
        }
        a[o] = v;
    }
}

// ------------------------------------------------------------------------------------------------
// eff: throughput of a tile shape relative to 128x128, measured on MFMA-bound layers with many
// workgroups per CU (smaller tiles move more operand bytes per MFMA and spend more issue slots on
// the gather).
// bf16 MFMA kernels (measured on the 3x3 64->192 layer at 56x56, batch 256): they are bound by the
// per-slab instruction overhead, not by the MFMA pipe, so 64-row tiles with many pixels win.
constexpr TileCfg kTilesBf16[] = {
    {64, 256, 1.00f}, {64, 128, 0.955f}, {64, 64, 0.83f}, {96, 256, 0.81f}, {32, 256, 0.77f},
    {32, 128, 0.77f}, {128, 128, 0.64f}, {96, 128, 0.58f}, {128, 64, 0.30f},
};
constexpr float kEff16 = 0.96f;   // 16x16x4 tiles, 256 pixels per workgroup (measured like the table below)
constexpr TileCfg kTiles[] = {
    {192, 128, 0.0f},   // only when forced, until calibrated
    {128, 128, 1.00f}, {96, 256, 0.85f}, {96, 128, 1.00f}, {64, 256, 0.85f}, {128, 64, 0.93f},
    {64, 128, 0.90f},  {32, 256, 0.78f}, {64, 64, 0.92f},  {32, 128, 0.80f},
};

template <typename T, bool MINUS, bool D2S, bool FUSED, int TM, int TN, int WM, int WN, int MT = 32>
hipError_t launch_tap(PixParams& p, hipStream_t st) {
    const bool buf = p.in_bytes != 0;
    const long long total = (long long)p.tiles_i * p.tiles_pix;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    if (buf)
        hipLaunchKernelGGL((igemm_tap_kernel<T, MINUS, D2S, FUSED, TM, TN, WM, WN, MT, true>), dim3((unsigned)total),
                           dim3(WM * WN * 64), 0, st, p);
    else
        hipLaunchKernelGGL((igemm_tap_kernel<T, MINUS, D2S, FUSED, TM, TN, WM, WN, MT, false>), dim3((unsigned)total),
                           dim3(WM * WN * 64), 0, st, p);
    return hipGetLastError();
}

template <typename T, bool FUSED, int TM, int TN, int WM, int WN>
hipError_t launch_flat(PixParams& p, hipStream_t st) {
    // no padding: every tap of every output pixel lies inside the image, no bounds tests needed
    const bool nopad = p.g_add_h == 0 && p.g_add_w == 0 &&
                       (p.Ho - 1) * p.g_mul_h + p.R <= p.Hi && (p.Wo - 1) * p.g_mul_w + p.S <= p.Wi;
    const long long total = (long long)p.tiles_i * p.tiles_pix;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    // two-part offsets: gathered tensor and filter below 2^30 bytes
    const bool buf = p.in_bytes != 0 && p.in_bytes < (1u << 30) && (long long)p.Co * p.Kg * 4 < (1LL << 30);
#define FLAT_LAUNCH(NOPAD_, BUF_)                                                                          \
    hipLaunchKernelGGL((igemm_flat_kernel<T, FUSED, NOPAD_, BUF_, TM, TN, WM, WN>), dim3((unsigned)total),     \
                       dim3(WM * WN * 64), 0, st, p)
    if (nopad) { if (buf) FLAT_LAUNCH(true, true); else FLAT_LAUNCH(true, false); }
    else       { if (buf) FLAT_LAUNCH(false, true); else FLAT_LAUNCH(false, false); }
#undef FLAT_LAUNCH
    return hipGetLastError();
}

template <typename T, bool MINUS, bool D2S, bool FUSED>
hipError_t dispatch_tap2(PixParams& p, int bm, int bn, hipStream_t st) {
    // 16-row granular tiles (16x16x4 MFMA): 48 or 16 rows, 256 or 128 pixels
    if (bm == 48 && bn == 256) return launch_tap<T, MINUS, D2S, FUSED, 3, 4, 1, 4, 16>(p, st);
    if (bm == 48 && bn == 128) return launch_tap<T, MINUS, D2S, FUSED, 3, 2, 1, 4, 16>(p, st);
    if (bm == 16 && bn == 256) return launch_tap<T, MINUS, D2S, FUSED, 1, 4, 1, 4, 16>(p, st);
    if (bm == 16 && bn == 128) return launch_tap<T, MINUS, D2S, FUSED, 1, 2, 1, 4, 16>(p, st);
#define CALL(TM, TN, WM, WN) launch_tap<T, MINUS, D2S, FUSED, TM, TN, WM, WN>(p, st)
    PURINE_TILE_SWITCH(CALL)
#undef CALL
}
template <typename T, bool MINUS, bool D2S>
hipError_t dispatch_tap(PixParams& p, int bm, int bn, hipStream_t st) {
    const bool fused = p.bias || p.relu || p.mask;
    return fused ? dispatch_tap2<T, MINUS, D2S, true>(p, bm, bn, st)
                 : dispatch_tap2<T, MINUS, D2S, false>(p, bm, bn, st);
}
template <typename T, bool FUSED>
hipError_t dispatch_flat2(PixParams& p, int bm, int bn, hipStream_t st) {
#define CALL(TM, TN, WM, WN) launch_flat<T, FUSED, TM, TN, WM, WN>(p, st)
    PURINE_TILE_SWITCH(CALL)
#undef CALL
}
template <typename T>
hipError_t dispatch_flat(PixParams& p, int bm, int bn, hipStream_t st) {
    const bool fused = p.bias || p.relu || p.mask;
    return fused ? dispatch_flat2<T, true>(p, bm, bn, st) : dispatch_flat2<T, false>(p, bm, bn, st);
}

}  // namespace

// Tile choice: every workgroup costs bm*bn/eff, where eff discounts the smaller tiles for their extra
// operand traffic per MFMA; the busiest of the 256 CUs gets ceil(workgroups/256) of them. Pick the
// tile that minimises that CU's load (padding waste is part of it, through the tile counts).
static int g_force_bm = 0, g_force_bn = 0;   // tuning hook, see purine_debug_force_tile
static int g_no_buffer_loads = 0;            // tuning hook: bn == -1 in purine_debug_force_tile
bool buffer_loads_disabled() { return g_no_buffer_loads != 0; }
bool patch_split_roles_disabled() { return g_force_bm == -4; }   // tuning hook: force_pix_tile(-4, x)
bool patch_split_roles_forced() { return g_force_bm == -5; }     // test hook: force_pix_tile(-5, x), also for layers of few tiles
void force_pix_tile(int bm, int bn) {
    g_no_buffer_loads = (bn == -1 && bm != -2) ? 1 : 0;
    g_force_bm = bm; g_force_bn = bn;
}

// Geometry of the implicit GEMM for one pass (everything in PixParams that does not depend on the
// tensors' addresses, the epilogue options or beta).
static PixParams make_pix_params(int dtype, const ConvGeom& g, const PixPlan& pl) {
    PixParams p{};
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W;
    p.sh = g.sh; p.sw = g.sw; p.ph = g.ph; p.pw = g.pw;
    p.R = g.R; p.S = g.S; p.RS = g.R * g.S;
    p.Ci = pl.Ci; p.Co = pl.Co; p.Rt = pl.Rt; p.St = pl.St;
    p.Ci_pad = pl.Ci_pad; p.i_pad = pl.i_pad;
    p.phases = 1;
    if (pl.mode == 0) {
        p.Hi = g.H; p.Wi = g.W; p.Ho = g.P; p.Wo = g.Q;
        p.g_mul_h = g.sh; p.g_mul_w = g.sw; p.g_add_h = -g.ph; p.g_add_w = -g.pw;
    } else if (pl.mode == 1) {
        p.Hi = g.P; p.Wi = g.Q; p.Ho = g.H; p.Wo = g.W;
        p.g_mul_h = 1; p.g_mul_w = 1; p.g_add_h = g.ph; p.g_add_w = g.pw;
    } else {
        // Strided backward-data, phase-folded. Write h + ph = hq*sh + a and w + pw = wq*sw + b.
        // Only taps r = a + sh*r', s = b + sw*s' reach such a position, from p = hq - r',
        // q = wq - s'. So dx is a unit-stride correlation of dy with ceil(R/sh) x ceil(S/sw) taps that
        // produces C*sh*sw "channels" (c, a, b) per coarse pixel (hq, wq), followed by a
        // depth-to-space shuffle in the epilogue. No multiply is spent on the structural zeros of
        // the strided transposed convolution, and the GEMM's row count grows from C to C*sh*sw.
        p.Hi = g.P; p.Wi = g.Q;
        p.phases = g.sh * g.sw;
        p.hq_min = g.ph / g.sh; p.wq_min = g.pw / g.sw;
        p.Ho = (g.H - 1 + g.ph) / g.sh - p.hq_min + 1;
        p.Wo = (g.W - 1 + g.pw) / g.sw - p.wq_min + 1;
        p.g_mul_h = 1; p.g_mul_w = 1; p.g_add_h = p.hq_min; p.g_add_w = p.wq_min;
    }
    p.HiWi = p.Hi * p.Wi;
    p.HoWo = p.Ho * p.Wo;
    p.M = p.N * p.HoWo;
    p.in_ns = pl.mode == 0 ? g.x_ns : g.y_ns;    // forward gathers x, backward-data gathers dy
    p.out_ns = pl.mode == 0 ? g.y_ns : g.x_ns;
    p.Kg = p.Ci * p.RS;
    p.div_howo = make_fastdiv(p.HoWo);
    p.div_wo = make_fastdiv(p.Wo);
    p.div_phases = make_fastdiv(p.phases);
    p.div_sw = make_fastdiv(p.sw);
    p.div_rs = make_fastdiv(p.RS);
    p.div_s = make_fastdiv(p.S);
    p.tiles_i = pl.tiles_i; p.tiles_pix = pl.tiles_pix;
    {
        // raw-buffer gather of the fp32 tap kernels: the whole tensor must be addressable with byte
        // offsets below 2^31
        const long long in_bytes = ((long long)(p.N - 1) * p.in_ns + (long long)p.Ci * p.HiWi) * 4;
        p.in_bytes = (dtype == PURINE_F32 && in_bytes < 0x7fffffffLL && g_no_buffer_loads == 0) ? (unsigned)in_bytes : 0u;
        // raw-buffer stores of the epilogues into an NCHW output (not the depth-to-space one)
        const long long out_bytes = ((long long)(p.N - 1) * p.out_ns + (long long)p.Co * p.HoWo) * (dtype == PURINE_BF16 ? 2 : 4);
        p.out_bytes = (pl.mode != 2 && out_bytes < 0x7fffffffLL && g_no_buffer_loads == 0) ? (unsigned)out_bytes : 0u;
    }

    return p;
}

PixPlan plan_conv_pix(const ConvGeom& g, bool bwd_data, int dtype, bool fused, bool accumulate) {
    PixPlan pl{};
    const int elem = dtype == PURINE_BF16 ? 2 : 4;
    int Co, Ci;
    long long M;
    if (!bwd_data) {
        pl.mode = 0; Co = g.K; Ci = g.C; M = (long long)g.N * g.P * g.Q;
        pl.Rt = g.R; pl.St = g.S;
    } else if (g.sh == 1 && g.sw == 1) {
        pl.mode = 1; Co = g.C; Ci = g.K; M = (long long)g.N * g.H * g.W;
        pl.Rt = g.R; pl.St = g.S;
    } else {
        pl.mode = 2; Co = g.C * g.sh * g.sw; Ci = g.K;
        const int Hq = (g.H - 1 + g.ph) / g.sh - g.ph / g.sh + 1;
        const int Wq = (g.W - 1 + g.pw) / g.sw - g.pw / g.sw + 1;
        M = (long long)g.N * Hq * Wq;
        pl.Rt = (g.R + g.sh - 1) / g.sh; pl.St = (g.S + g.sw - 1) / g.sw;
    }
    pl.flat = !bwd_data && Ci < BK && (dtype == PURINE_BF16 || Ci * g.R * g.S <= FLAT_MAX_KG);
    // Time model per tile shape: workgroups are dealt round-robin to the 256 CUs and a CU's MFMA pipe
    // is shared by whatever it holds, so the kernel lasts as long as the busiest CU:
    // ceil(workgroups/256) * bm*bn/eff. A CU holding one or two workgroups has too few wavefronts to
    // hide memory latency (measured: about 5% and 40% slower). Every row tile gathers its pixel
    // columns again, which matters for the flat kernel, whose gather decodes (c,r,s) per row.
    (void)fused;
    const double gather = pl.flat ? 15.0 : 3.0;
    double best = -1.0;
    // the bf16 modes that gather single 2-byte elements (flattened, and single-tap straight from NCHW)
    const bool flat_bf16 = dtype == PURINE_BF16 && (pl.flat || pl.Rt * pl.St == 1);
    const TileCfg* table = dtype == PURINE_BF16 ? kTilesBf16 : kTiles;
    const int n_table = dtype == PURINE_BF16 ? (int)(sizeof(kTilesBf16) / sizeof(TileCfg)) : (int)(sizeof(kTiles) / sizeof(TileCfg));
    for (int ti_ = 0; ti_ < n_table; ++ti_) {
        const TileCfg& t = table[ti_];
        if (t.eff <= 0.0f) continue;
        const long long ti = (Co + t.bm - 1) / t.bm, tp = (M + t.bn - 1) / t.bn;
        const long long per_cu = (ti * tp + 255) / 256;
        const double hide = per_cu >= 3 ? 1.0 : (per_cu == 2 ? 0.95 : 0.6);
        // the bf16 element-gather modes fetch 32 elements per thread and slab at 256 pixels per
        // workgroup, which measured a third slower than 16 at 128
        // ... and in a single-tap bf16 layer 64 pixels per workgroup measured faster again than 128
        // (64 -> 64 channels at 56x56 with the pixel-pair gather: forward 0.055 -> 0.048 ms,
        // backward-data 0.045 -> 0.043 ms)
        const double eff = (flat_bf16 && t.bn == 256) ? t.eff * 0.65
                         : (flat_bf16 && !pl.flat && t.bm == 64 && t.bn == 64) ? 1.04 : t.eff;
        const double load = (double)per_cu * t.bm * t.bn * (1.0 + gather / t.bm) / (eff * hide);
        if (best < 0 || load < best) { best = load; pl.bm = t.bm; pl.bn = t.bn; }
    }
    // GEMMs with at most 16, or 33..48, rows (first-layer backward-data after phase folding): tiles of
    // 16x16x4 MFMAs waste no half tile of rows
    const bool rows16 = dtype == PURINE_F32 && !pl.flat && (Co <= 16 || (Co > 32 && Co <= 48) || (Co > 80 && Co <= 96));
    if (rows16) {
        const int bm16 = Co <= 16 ? 16 : 48;
        for (int bn16 = 256; bn16 >= 128; bn16 /= 2) {
            const long long per_cu = ((Co + bm16 - 1) / bm16 * ((M + bn16 - 1) / bn16) + 255) / 256;
            const double hide = per_cu >= 3 ? 1.0 : (per_cu == 2 ? 0.95 : 0.6);
            const double eff = bn16 == 256 ? kEff16 : kEff16 * 0.96;
            const double load = (double)per_cu * bm16 * bn16 * (1.0 + gather / bm16) / (eff * hide);
            if (load < best) { best = load; pl.bm = bm16; pl.bn = bn16; }
        }
    }
    for (const TileCfg& t : kTiles)
        if (t.bm == g_force_bm && t.bn == g_force_bn) { pl.bm = t.bm; pl.bn = t.bn; }
    if (rows16 && (g_force_bn == 256 || g_force_bn == 128) && g_force_bm == (Co <= 16 ? 16 : 48)) {
        pl.bm = g_force_bm; pl.bn = g_force_bn;
    }
    pl.Co = Co; pl.Ci = Ci;
    pl.tiles_i = (Co + pl.bm - 1) / pl.bm;
    pl.tiles_pix = (int)((M + pl.bn - 1) / pl.bn);
    const int depth = dtype == PURINE_BF16 ? 32 : BK;   // slab depth of the kernel that will run
    // the bf16 flattened kernel reads a padded filter copy A[i][C*R*S rounded up]
    const bool flat_copy = pl.flat && dtype == PURINE_BF16;
    const int red = flat_copy ? Ci * g.R * g.S : Ci;
    pl.Ci_pad = (red + depth - 1) / depth * depth;
    pl.i_pad = pl.tiles_i * pl.bm;
    // scratch is sized for the widest row padding any tile shape could ask for (96- or 128-row
    // tiles), so the size does not depend on which shape, plain or fused, ends up running
    const long long pad96 = (long long)(Co + 95) / 96 * 96, pad128 = (long long)(Co + 127) / 128 * 128;
    const long long pad192 = (long long)(Co + 191) / 192 * 192;
    long long i_pad_max = pad96 > pad128 ? pad96 : pad128;
    if (pad192 > i_pad_max) i_pad_max = pad192;
    pl.ws_bytes = flat_copy ? (size_t)pl.Ci_pad * (size_t)i_pad_max * elem
                  : pl.flat ? 0 : (size_t)pl.Rt * pl.St * pl.Ci_pad * (size_t)i_pad_max * elem;
    if (flat_copy) {   // the row-staging kernel's filter copy can be the larger one (short filter rows)
        const size_t rows_bytes = rows_filter_bytes(g.K, g.C, g.R, g.S);
        if (rows_bytes > pl.ws_bytes) pl.ws_bytes = rows_bytes;
    }
    pl.blk_offset = 0;
    pl.patch = false;
    if (dtype == PURINE_BF16 && !pl.flat && pl.Rt * pl.St > 1 && g_force_bm != -2) {
        // layers whose gathered rows are whole 16-byte packets and whose gather has unit stride stage
        // the input patch in LDS and need no re-laid-out copy (tuning hook: force_pix_tile(-2, x) keeps
        // them on the blocked-copy kernel)
        PixParams probe = make_pix_params(dtype, g, pl);
        PatchGeom q;
        pl.patch = plan_patch_bf16(probe, pl.mode, &q);
        if (pl.patch) pl.ws_bytes = patch_filter_bytes(Co, Ci, pl.Rt * pl.St);
    }
    if (dtype == PURINE_BF16 && !pl.flat && pl.Rt * pl.St > 1 && !pl.patch) {
        // channels-blocked copy of the gathered tensor behind the filter copy (single-tap layers
        // gather each element once, straight from NCHW)
        const size_t gathered = (size_t)g.N * pl.Ci_pad * (bwd_data ? (size_t)g.P * g.Q : (size_t)g.H * g.W);
        pl.blk_offset = (pl.ws_bytes + 255) / 256 * 256;
        pl.ws_bytes = pl.blk_offset + gathered * elem;
    }
    // identity gather: the streaming GEMM applies
    const long long HW = (long long)g.H * g.W;
    const bool forced = (g_force_bn == 1 || g_force_bn == 2 || g_force_bn == 4) && g_force_bm >= 32 &&
                        g_force_bm <= 96 && g_force_bm % 32 == 0 && HW % g_force_bn == 0 &&
                        !(g_force_bn == 4 && g_force_bm == 96) && !(g_force_bn == 1 && g_force_bm == 32);
    // bf16 layers do better on the bf16 MFMA kernel: they take this one only when told to
    pl.gemm1x1 = g.R == 1 && g.S == 1 && g.sh == 1 && g.sw == 1 && g.ph == 0 && g.pw == 0 &&
                 Ci >= 16 && Ci % 16 == 0 && HW % 2 == 0 && g_force_bm != -1 &&
                 (dtype == PURINE_F32 || forced);
    if (pl.gemm1x1) {
        // One row tile of 96 that covers every output channel reads the activations once; otherwise
        // 32-row tiles with four pixels per lane (16-byte loads and stores) measured best, the
        // repeated activation reads being served by L2.
        // The backward pass through a ReLU mask also reads the mask tensor in its epilogue: there
        // 32-row tiles with two pixels per lane measured 9 % faster than the 96-row tile (more,
        // shorter workgroups overlap the mask reads and stores of one with the streaming of others).
        if (Co > 64 && Co <= 96 && !(bwd_data && fused)) { pl.gemm_tm = 3; pl.gemm_tn = 2; }
        else if (Co > 64 && Co <= 96) { pl.gemm_tm = 1; pl.gemm_tn = 2; }
        else { pl.gemm_tm = 1; pl.gemm_tn = HW % 4 == 0 ? 4 : 2; }
        // An accumulating backward-data pass (dx += ...) reads the old dx in its epilogue, like the
        // mask above: two pixels per lane again (the inception module's merged 1x1, 192 rows:
        // 0.098 -> 0.086 ms). Only where the reduction is too short to be split (the scratch size
        // is asked for without knowing whether the call will accumulate).
        if (bwd_data && accumulate && !fused && (Ci + 127) / 128 < 4 && dtype == PURINE_F32) { pl.gemm_tm = 1; pl.gemm_tn = 2; }
        if (forced) { pl.gemm_tm = g_force_bm / 32; pl.gemm_tn = g_force_bn; }
        pl.gemm_tiles_i = (Co + pl.gemm_tm * 32 - 1) / (pl.gemm_tm * 32);
        pl.gemm_tiles_pix = (int)((M + 4 * 32 * pl.gemm_tn - 1) / (4 * 32 * pl.gemm_tn));
        // Too few tiles for 256 CUs and a long reduction (fully-connected backward-data: 128 rows x 9216
        // pixels over 4096 channels = 72 tiles): split the channels in whole 128-channel filter stages
        // so that about 2.5 workgroups per CU run, fp32 partial tiles behind the filter copy.
        pl.gemm_splits = 1; pl.gemm_split_ci = Ci; pl.gemm_part_offset = 0;
        const long long tiles = (long long)pl.gemm_tiles_i * pl.gemm_tiles_pix;
        const int stages = (Ci + 127) / 128;
        if (tiles < 320 && stages >= 4 && g_force_bm != -3) {
            // stages per split: the kernel lasts (workgroups of the busiest CU) x (stages per workgroup),
            // the second pass about 0.15 of a stage per split; at least two stages per split
            int per = stages;
            double best_t = -1.0;
            for (int c = stages; c >= 2; --c) {
                const int sp = (stages + c - 1) / c;
                const long long rounds = (tiles * sp + 255) / 256;
                const double t = (double)rounds * c + 0.15 * sp;
                if (best_t < 0 || t < best_t) { best_t = t; per = c; }
            }
            const int splits = (stages + per - 1) / per;
            const unsigned long long part = (unsigned long long)splits * (unsigned long long)g.N * Co * HW * 4ull;
            if (splits > 1 && part <= (256ull << 20)) {
                pl.gemm_splits = splits; pl.gemm_split_ci = per * 128;
                pl.gemm_part_offset = (pl.ws_bytes + 255) / 256 * 256;
                pl.ws_bytes = pl.gemm_part_offset + (size_t)part;
            }
        }
    }
    return pl;
}

hipError_t launch_conv_pix(int dtype, const ConvGeom& g, const PixPlan& pl, const void* in,
                           const void* wt, void* out, float beta, void* ws, const PixEpilogue& epi,
                           hipStream_t st) {
    PixParams p = make_pix_params(dtype, g, pl);
    p.in = in; p.out = out;
    p.bias = epi.bias; p.relu = epi.relu; p.mask = epi.mask;
    p.beta = beta;

    if (pl.gemm1x1) {
        const uintptr_t align = (uintptr_t)pl.gemm_tn * (dtype == PURINE_BF16 ? 2 : 4) - 1;
        if ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)epi.mask) & align) == 0) {
            PixParams q = p;
            q.wt = wt;
            q.tiles_i = pl.gemm_tiles_i; q.tiles_pix = pl.gemm_tiles_pix;
            if (pl.gemm_splits > 1) {
                if (!ws) return hipErrorInvalidValue;
                q.splits = pl.gemm_splits; q.split_ci = pl.gemm_split_ci;
                q.partial = (float*)((char*)ws + pl.gemm_part_offset);
            }
            return dispatch_gemm1x1(q, dtype, pl.mode == 1, pl.gemm_tm, pl.gemm_tn, st);
        }
    }
    if (pl.flat && dtype == PURINE_BF16 && g_force_bm != -2) {
        // input rows staged in LDS (rows of whole 16-byte packets); otherwise the flattened gather below
        RowsGeom rq;
        PixParams pr = p;
        if (plan_rows_bf16(pr, &rq)) {
            if (!ws) return hipErrorInvalidValue;
            ProbeScope whole_op(st, true);
            return launch_rows_bf16(pr, rq, wt, ws, st);
        }
    }
    if (pl.flat && dtype == PURINE_BF16) {
        // bf16 MFMA on the flattened reduction: padded filter copy A[i][Kg_pad] into scratch first
        RepackParams q{};
        q.w = wt; q.a = ws; q.mode = 3;
        q.K = g.K; q.C = g.C; q.R = g.R; q.S = g.S; q.sh = g.sh; q.sw = g.sw;
        q.St = 1; q.Ci = p.Kg; q.Co = pl.Co; q.Ci_pad = pl.Ci_pad; q.i_pad = pl.i_pad;
        const long long total = (long long)pl.Ci_pad * pl.i_pad;
        if (total > 0x7fffffffLL || !ws) return hipErrorInvalidValue;
        q.total = (int)total;
        q.i_major = 1;
        const unsigned blocks = (unsigned)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
        (void)hipGetLastError();
        hipLaunchKernelGGL(repack_filter_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, q);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
        p.wt = ws;
        p.Rt = 1; p.St = 1;
        return dispatch_flat_bf16(p, pl.bm, pl.bn, st);
    }
    if (pl.flat) {
        p.wt = wt;
        return dispatch_flat<float>(p, pl.bm, pl.bn, st);   // bf16 took the branch above
    }
    // bf16: the whole operator (input copy, filter repack, main kernel) is what a timing probe brackets
    ProbeScope whole_op(dtype == PURINE_BF16 ? st : nullptr, dtype == PURINE_BF16);
    if (pl.patch) {
        PatchGeom qg;
        if (!plan_patch_bf16(p, pl.mode, &qg) || !ws) return hipErrorInvalidValue;
        hipError_t e = repack_patch_filter(p, pl.mode, wt, ws, g.K, g.C, st);
        if (e != hipSuccess) return e;
        p.wt = ws;
        return launch_patch_bf16(p, qg, pl.mode, st);
    }
    const bool blocked = dtype == PURINE_BF16 && pl.Rt * pl.St > 1;
    if (blocked) {
        if (!pl.blk_offset || !ws) return hipErrorInvalidValue;
        hipError_t e = blockify_input(p, (char*)ws + pl.blk_offset, st);
        if (e != hipSuccess) return e;
    }
    // repack the filter into scratch, then run the tap-major kernel on it
    RepackParams q{};
    q.w = wt; q.a = ws; q.mode = pl.mode;
    q.K = g.K; q.C = g.C; q.R = g.R; q.S = g.S; q.sh = g.sh; q.sw = g.sw;
    q.St = pl.St; q.Ci = pl.Ci; q.Co = pl.Co; q.Ci_pad = pl.Ci_pad; q.i_pad = pl.i_pad;
    const long long total = (long long)pl.Rt * pl.St * pl.Ci_pad * pl.i_pad;
    if (total > 0x7fffffffLL) return hipErrorInvalidValue;
    q.total = (int)total;
    q.i_major = dtype == PURINE_BF16 ? 1 : 0;
    {
        const unsigned blocks = (unsigned)((total + 255) / 256 > 4096 ? 4096 : (total + 255) / 256);
        (void)hipGetLastError();
        if (dtype == PURINE_F32)
            hipLaunchKernelGGL(repack_filter_kernel<float>, dim3(blocks), dim3(256), 0, st, q);
        else
            hipLaunchKernelGGL(repack_filter_kernel<uint16_t>, dim3(blocks), dim3(256), 0, st, q);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    p.wt = ws;
    if (dtype == PURINE_F32) {
        if (pl.mode == 0) return dispatch_tap<float, false, false>(p, pl.bm, pl.bn, st);
        if (pl.mode == 1) return dispatch_tap<float, true, false>(p, pl.bm, pl.bn, st);
        return dispatch_tap<float, true, true>(p, pl.bm, pl.bn, st);
    }
    return blocked ? dispatch_tap_bf16(p, pl.mode, pl.bm, pl.bn, st)
                   : dispatch_tap_bf16_nchw(p, pl.mode, pl.bm, pl.bn, st);
}

}  // namespace purine

// Device-side pieces shared by the forward / backward-data implicit-GEMM kernels (fp32 and bf16 MFMA).
#pragma once
#include "common.h"
#include <type_traits>

namespace purine {
namespace pix {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

// Accumulator of one MFMA tile and the matching fp32 instruction: 32x32x2 (16 values per lane) or
// 16x16x4 (4 values per lane).
template <int MT> struct AccT;
template <> struct AccT<32> {
    typedef floatx16 type;
    static constexpr int N = 16;
    static __device__ __forceinline__ type mfma(float a, float b, type c) {
        return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0);
    }
};
template <> struct AccT<16> {
    typedef floatx4 type;
    static constexpr int N = 4;
    static __device__ __forceinline__ type mfma(float a, float b, type c) {
        return __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, c, 0, 0, 0);
    }
};

template <typename T> struct Elem;
template <> struct Elem<float> {
    static __device__ __forceinline__ float load(const float* p, int i) { return p[i]; }
    static __device__ __forceinline__ void store(float* p, int i, float v) { p[i] = v; }
    static __device__ __forceinline__ floatx4 load4(const float* p, int i) {
        return *reinterpret_cast<const floatx4*>(p + i);
    }
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
    static __device__ __forceinline__ floatx4 load4(const uint16_t* p, int i) {
        const uint2 v = *reinterpret_cast<const uint2*>(p + i);
        floatx4 o;
        o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xffff0000u);
        o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xffff0000u);
        return o;
    }
};

// Longest flattened reduction C*R*S the fp32 flat forward kernel keeps a row table for (a multiple of
// the slab depth); longer ones take the tap-major kernel.
constexpr int FLAT_MAX_KG = 2048;

struct PixParams {
    const void* in;     // gathered activation tensor [N][Ci][Hi][Wi]
    const void* wt;     // tap kernel: repacked filter A[taps][Ci_pad][i_pad]; flat kernel: KCRS filter
    void* out;          // produced tensor [N][Co][Ho][Wo] (depth-to-space epilogue: dx [N][C][H][W])
    int N, Ci, Hi, Wi, HiWi;
    int Co, Ho, Wo, HoWo, M;      // GEMM rows; pixel grid enumerated by the columns; M = N*Ho*Wo
    int Rt, St;                   // taps of the reduction (ceil(R/sh) x ceil(S/sw) when phase-folded)
    int Ci_pad, i_pad;            // padded extents of the repacked filter
    int g_mul_h, g_mul_w, g_add_h, g_add_w;   // gather origin: g_h = ho*g_mul_h + g_add_h (same for w)
    int C, H, W, sh, sw, ph, pw, phases, hq_min, wq_min;   // depth-to-space epilogue
    int R, S, RS, Kg;             // flat kernel only: filter extents, Kg = Ci*R*S
    FastDiv div_howo, div_wo, div_phases, div_sw, div_rs, div_s;
    float beta;
    // fused epilogue (all optional): out = relu?(acc + bias[row]) and/or out = (mask[o] > 0 ? acc : 0)
    const void* bias;   // [Co], same dtype as out; forward only
    const void* mask;   // same extents and dtype as out: ReLU output whose gradient this pass produces
    int relu;
    int tiles_i, tiles_pix;
    unsigned in_bytes;   // span of the gathered tensor when the fp32 tap kernels may read it as a raw buffer, else 0
    unsigned out_bytes;  // span of the NCHW output when the epilogues may write it as a raw buffer (below 2^31 bytes), else 0
    // elements between consecutive images of the gathered and of the produced tensor (the mask shares
    // the latter): Ci*Hi*Wi and the dense image size of `out` unless they are channel-slice views
    int in_ns, out_ns;
    // split reduction of the 1x1 streaming GEMM (GEMMs with too few tiles to fill the chip): blockIdx.y
    // takes `split_ci` gathered channels and writes a raw fp32 tile into partial[split][N][Co][Ho*Wo];
    // a second kernel adds the splits in a fixed order and applies the epilogue. splits <= 1: off.
    int splits, split_ci;
    float* partial;
};

typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
typedef float floatx2 __attribute__((ext_vector_type(2)));

// Two fp32 values to two bf16 (round to nearest even) in one dword, first value in the low half.
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    const floatx2 f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2));
}
// The fused forward kernels stage their row tile's bias values in LDS at kernel start (zero past the
// last output channel), so the epilogue does not wait on global memory for them. The caller's
// first barrier orders the fill before any use.
template <typename T, int BM, int NT>
__device__ __forceinline__ void stage_bias(float* bias_lds, const PixParams& p, int i0, int tid) {
    const T* __restrict__ bias = (const T*)p.bias;
    if (bias)
        for (int r = tid; r < BM; r += NT) bias_lds[r] = i0 + r < p.Co ? Elem<T>::load(bias, i0 + r) : 0.0f;
}

// Epilogue shared by the kernels (pix_limit: columns at or past this pixel index are not stored;
// kernels whose pixel tiles stop at image boundaries pass the end of their image. bstep: distance in
// pixels between a lane's consecutive column tiles: 32, or 1 for kernels that give a lane adjacent pixels).
// Accumulator register e of a 32x32 tile holds row
// (e/4)*8 + (lane/32)*4 + e%4, column lane%32. Optional pieces (bias, ReLU, ReLU-gradient mask,
// accumulate) are uniform branches; what an element needs from memory (mask value, old output) is
// fetched for a batch of rows of one MFMA tile BEFORE their stores, so the loads overlap instead of
// forming load-wait-store round trips, while few extra registers are live.
template <typename T, bool D2S>
struct TileAddr {
    const PixParams& p;
    int obase, hb, wb;
    __device__ __forceinline__ TileAddr(const PixParams& p_, int n, int rem) : p(p_), hb(0), wb(0) {
        if (!D2S) {
            obase = n * p.out_ns + rem;
        } else {
            // depth-to-space: row i = (c, a, b) of coarse pixel (n, hq, wq) is
            // dx[n, c, hq*sh + a - ph, wq*sw + b - pw]
            const int hq = fastdiv(rem, p.div_wo);
            const int wq = rem - hq * p.Wo;
            hb = (hq + p.hq_min) * p.sh - p.ph;
            wb = (wq + p.wq_min) * p.sw - p.pw;
            obase = n * p.out_ns;
        }
    }
    // element offset of row i (0 when the row or position does not exist) and whether it exists
    __device__ __forceinline__ int at(int i, bool& ok) const {
        int off;
        if (!D2S) {
            ok = i < p.Co;
            off = obase + i * p.HoWo;
        } else {
            const int c = fastdiv(i, p.div_phases);
            const int ab = i - c * p.phases;
            const int pa = fastdiv(ab, p.div_sw);
            const int pb = ab - pa * p.sw;
            const int h = hb + pa, w = wb + pb;
            ok = (i < p.Co) & ((unsigned)h < (unsigned)p.H) & ((unsigned)w < (unsigned)p.W);
            off = obase + (c * p.H + h) * p.W + w;
        }
        return ok ? off : 0;
    }
};

// FWD: the forward pass (bias / ReLU may be fused, never a mask or an accumulate); otherwise
// backward-data (mask and accumulate possible, never bias / ReLU). Knowing the pass at compile time
// keeps the other pass's options out of the per-element code.
template <typename T, bool D2S, bool FUSED, int TM, int TN, bool FWD>
__device__ __forceinline__ void store_tile(const PixParams& p, T* __restrict__ out,
                                           floatx16 (&acc)[TM][TN], int i_base, int pix_base,
                                           int khalf, const float* bias_lds, int i_tile0,
                                           int pix_limit = 0x7fffffff, int bstep = 32) {
    if ((!FUSED || FWD) && !D2S && p.out_bytes != 0) {
        // NCHW output through raw buffer stores: a lane's pixel (and its half's four rows) is one
        // offset register per column tile, set up once; a row's part of the address is a scalar; a
        // row at or past Co gets an offset outside the resource and the hardware drops the store.
        // (With plain pointers every element carried its own row test and exec-mask branch, a 64-bit
        // address computation and, for a fused bias, an LDS round trip of its own: over twenty
        // instructions per store.)
        const bool fwd_bias = FUSED && FWD && p.bias != nullptr, fwd_relu = FUSED && FWD && p.relu;
        const bool has_beta = !FWD && p.beta != 0.0f;
        const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc(out, (short)0, (int)p.out_bytes, 0x00020000);
        unsigned voff[TN];
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int pix = pix_base + b * bstep;
            const bool live = pix < p.M && pix < pix_limit;
            const int n = fastdiv(live ? pix : 0, p.div_howo);
            voff[b] = live ? (unsigned)(n * p.out_ns + (pix - n * p.HoWo) + khalf * 4 * p.HoWo) * (unsigned)sizeof(T) : 0x80000000u;
        }
        const int rows0 = __builtin_amdgcn_readfirstlane(i_base);
        auto rows = [&](auto relu_c) {
            constexpr bool RELU = decltype(relu_c)::value;
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                floatx4 bq = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int row_lo = rows0 + a * 32 + (e >> 2) * 8 + (e & 3);     // scalar; this lane's row is khalf * 4 further
                    if (row_lo >= p.Co) continue;                                   // uniform
                    const int soff = row_lo * p.HoWo * (int)sizeof(T);
                    const bool row_ok = row_lo + khalf * 4 < p.Co;
                    float bv = 0.0f;
                    if (FUSED && FWD && sizeof(T) == 2) {
                        // bf16 kernels are short per wavefront: the bias of the four consecutive rows of an
                        // accumulator quad comes as one 16-byte LDS read instead of four round trips
                        if ((e & 3) == 0 && fwd_bias) bq = *reinterpret_cast<const floatx4*>(&bias_lds[row_lo + khalf * 4 - i_tile0]);
                        bv = bq[e & 3];
                    } else if (FUSED && FWD) {
                        bv = fwd_bias ? bias_lds[row_lo + khalf * 4 - i_tile0] : 0.0f;
                    }
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        const unsigned vo = row_ok ? voff[b] : 0x80000000u;
                        float v = acc[a][b][e];
                        if (FUSED && FWD) v += bv;
                        if (RELU) v = v > 0.0f ? v : 0.0f;
                        if (sizeof(T) == 4) {
                            if (has_beta) v += __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(r_out, vo, soff, 0));
                            __builtin_amdgcn_raw_buffer_store_b32(__builtin_bit_cast(uint32_t, v), r_out, vo, soff, 0);
                        } else {
                            if (has_beta) v += __uint_as_float((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r_out, vo, soff, 0) << 16);
                            __builtin_amdgcn_raw_buffer_store_b16((uint16_t)(pack_bf16(v, 0.0f) & 0xffffu), r_out, vo, soff, 0);
                        }
                    }
                }
            }
        };
        if (fwd_relu) rows(std::true_type{}); else rows(std::false_type{});
        return;
    }
    if (!FUSED || FWD) {
        // Plain store (backward-data: optionally accumulating) and the fused forward epilogue, which
        // needs nothing from global memory (bias comes from LDS): no staging arrays, so these
        // kernels keep their register count and occupancy. (Depth-to-space outputs, and NCHW outputs
        // of 2^31 bytes or more.)
        const bool fwd_bias = FUSED && FWD && !D2S && p.bias != nullptr, fwd_relu = FUSED && FWD && p.relu;
        constexpr bool QUAD = sizeof(T) == 2;   // bf16: bias of four consecutive rows as one 16-byte LDS read
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int pix = pix_base + b * bstep;
            if (pix >= p.M || pix >= pix_limit) continue;
            const int n = fastdiv(pix, p.div_howo);
            const TileAddr<T, D2S> addr(p, n, pix - n * p.HoWo);
#pragma unroll
            for (int a = 0; a < TM; ++a) {
                floatx4 bq = {0.0f, 0.0f, 0.0f, 0.0f};
                // The fused arithmetic needs the values in VGPRs (the plain store takes them from the
                // accumulator register file). Pinning the copy of ONE tile here, behind a fence, keeps
                // the compiler from copying every tile's accumulators out at once (96 VGPRs for a
                // six-tile wavefront, and a workgroup of occupancy with them).
                floatx16 tile = acc[a][b];
                if (FUSED) {
                    __builtin_amdgcn_sched_barrier(0);
                    asm volatile("" : "+v"(tile));
                }
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    bool ok;
                    const int row = i_base + a * 32 + khalf * 4 + (e >> 2) * 8 + (e & 3);
                    const int off = addr.at(row, ok);
                    if (QUAD && fwd_bias && (e & 3) == 0) bq = *reinterpret_cast<const floatx4*>(&bias_lds[row - i_tile0]);
                    if (ok) {
                        float v = tile[e];
                        if (fwd_bias) v += QUAD ? bq[e & 3] : bias_lds[row - i_tile0];
                        if (fwd_relu) v = v > 0.0f ? v : 0.0f;
                        if (!FWD && p.beta != 0.0f) v += Elem<T>::load(out, off);
                        Elem<T>::store(out, off, v);
                    }
                }
            }
        }
        return;
    }
    const T* __restrict__ bias = (const T*)p.bias;
    const T* __restrict__ mask = (const T*)p.mask;
    const bool has_bias = FWD && !D2S && bias != nullptr, has_mask = !FWD && mask != nullptr;
    const bool has_beta = !FWD && p.beta != 0.0f, relu = FWD && p.relu;
    constexpr int G = 4;   // rows per staged batch: one accumulator quad (16 rows cost the 96x128 kernel two wavefronts of occupancy)
    constexpr bool QUAD_BIAS = sizeof(T) == 2;
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int pix = pix_base + b * bstep;
        if (pix >= p.M || pix >= pix_limit) continue;
        const int n = fastdiv(pix, p.div_howo);
        const TileAddr<T, D2S> addr(p, n, pix - n * p.HoWo);
#pragma unroll
        for (int ag = 0; ag < TM * (16 / G); ++ag) {
            // The mask / old output values of G rows of an MFMA tile are requested before the first
            // of their stores, so that their latency is paid once per batch.
            const int a = ag / (16 / G), e0 = (ag % (16 / G)) * G;
            const int rowa = i_base + a * 32 + khalf * 4;
            float t[G], o[G];
            floatx4 bq = {0.0f, 0.0f, 0.0f, 0.0f};
            bool ok;
            if (has_mask && !has_bias) {
#pragma unroll
                for (int e = 0; e < G; ++e) t[e] = Elem<T>::load(mask, addr.at(rowa + ((e0 + e) >> 2) * 8 + (e & 3), ok));
            }
            if (has_beta) {
#pragma unroll
                for (int e = 0; e < G; ++e) o[e] = Elem<T>::load(out, addr.at(rowa + ((e0 + e) >> 2) * 8 + (e & 3), ok));
            }
#pragma unroll
            for (int e = 0; e < G; ++e) {
                const int row = rowa + ((e0 + e) >> 2) * 8 + (e & 3);
                const int off = addr.at(row, ok);
                float v = acc[a][b][e0 + e];
                // bias. bf16 kernels (short per wavefront, so the epilogue weighs): the four consecutive
                // rows e..e+3 of an accumulator quad come from LDS as one 16-byte read, instead of a read
                // per element that waits for its own round trip between two stores. The fp32 kernels
                // keep the per-element read: the quads cost the flattened forward kernel 20 registers
                // and with them a wavefront of occupancy.
                if (QUAD_BIAS) {
                    if (has_bias && (e & 3) == 0) bq = *reinterpret_cast<const floatx4*>(&bias_lds[row - i_tile0]);
                    if (has_bias) v += bq[e & 3];
                } else if (has_bias) {
                    v += bias_lds[row - i_tile0];
                }
                if (relu) v = v > 0.0f ? v : 0.0f;
                if (has_mask && !has_bias) v = t[e] > 0.0f ? v : 0.0f;
                if (has_beta) v += o[e];
                if (ok) Elem<T>::store(out, off, v);
            }
            // keep the next batch's loads from being hoisted above these stores
            __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Same epilogue for 16x16 MFMA tiles: accumulator register e holds row (lane/16)*4 + e, column
// lane%16; `kq` is lane/16.
template <typename T, bool D2S, bool FUSED, int TM, int TN, bool FWD>
__device__ __forceinline__ void store_tile(const PixParams& p, T* __restrict__ out,
                                           floatx4 (&acc)[TM][TN], int i_base, int pix_base, int kq,
                                           const float* bias_lds, int i_tile0) {
    const T* __restrict__ bias = (const T*)p.bias;
    const T* __restrict__ mask = (const T*)p.mask;
    const bool has_bias = FUSED && FWD && !D2S && bias != nullptr, has_mask = FUSED && !FWD && mask != nullptr;
    const bool has_beta = !FWD && p.beta != 0.0f, relu = FUSED && FWD && p.relu;
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int pix = pix_base + b * 16;
        if (pix >= p.M) continue;
        const int n = fastdiv(pix, p.div_howo);
        const TileAddr<T, D2S> addr(p, n, pix - n * p.HoWo);
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            const int row0 = i_base + a * 16 + kq * 4;
            float t[4], o[4];
            bool ok;
            if (D2S && sizeof(T) == 4 && !FUSED) {
                // stride-4 columns: the lane's four rows are four consecutive positions of one output
                // row (b = 0..3), written as one 16-byte packet (4-byte aligned) when all of them exist
                bool ok0, ok3;
                const int off0 = addr.at(row0, ok0);
                (void)addr.at(row0 + 3, ok3);
                if (p.sw == 4 && !has_beta && ok0 && ok3) {
                    typedef float floatx4_u __attribute__((ext_vector_type(4), aligned(4)));
                    floatx4_u v = {acc[a][b][0], acc[a][b][1], acc[a][b][2], acc[a][b][3]};
                    *reinterpret_cast<floatx4_u*>(reinterpret_cast<float*>(out) + off0) = v;
                    continue;
                }
            }
            if (has_bias) {
#pragma unroll
                for (int e = 0; e < 4; ++e) t[e] = bias_lds[row0 + e - i_tile0];
            } else if (has_mask) {
#pragma unroll
                for (int e = 0; e < 4; ++e) t[e] = Elem<T>::load(mask, addr.at(row0 + e, ok));
            }
            if (has_beta) {
#pragma unroll
                for (int e = 0; e < 4; ++e) o[e] = Elem<T>::load(out, addr.at(row0 + e, ok));
            }
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const int off = addr.at(row0 + e, ok);
                float v = acc[a][b][e];
                if (has_bias) v += t[e];
                if (relu) v = v > 0.0f ? v : 0.0f;
                if (has_mask) v = t[e] > 0.0f ? v : 0.0f;
                if (has_beta) v += o[e];
                if (ok) Elem<T>::store(out, off, v);
            }
        }
    }
}

// Epilogue for kernels whose lanes own TN ADJACENT pixels (column tile b of lane l is pixel
// TN * (l % 32) + b of the wavefront's strip) and NCHW bf16 outputs in which such a run is aligned
// (HoWo and the image distance multiples of TN): a lane writes its TN pixels of one row as one 4- or
// 8-byte packet, so the 32 lanes of a half-wavefront cover 32 * TN consecutive pixels of one row,
// whole 128-byte lines, and the fp32 -> bf16 conversion is the packed hardware one. Mask and old
// values are read the same way.
// The stores (and those reads) are raw buffer accesses on a resource that covers exactly image n's
// Co output rows: the lane's part of the address (its pixel, its half's four rows) is one VGPR set
// up once, the row's part a scalar, and a row at or past Co falls outside the resource and is dropped
// by the hardware. With plain pointers every store carried a 64-bit multiply-add, a row test with
// its exec-mask branch and the option flags' selects, about thirty instructions per store, and the
// epilogue of a 3x3 tile took as long as its MFMAs.
template <bool FUSED, int TM, int TN, bool FWD>
__device__ __forceinline__ void store_adjacent(const PixParams& p, floatx16 (&acc)[TM][TN], int i_base, int n,
                                               int pix_first, int pix_end, int lane, const float* bias_lds,
                                               int i_tile0) {
    static_assert(TN == 2 || TN == 4, "4- or 8-byte packets");
    typedef uint32_t packet_t __attribute__((ext_vector_type(TN / 2)));
    const bool has_bias = FUSED && FWD && p.bias != nullptr, relu = FUSED && FWD && p.relu;
    const bool has_mask = FUSED && !FWD && p.mask != nullptr, has_beta = !FWD && p.beta != 0.0f;
    const int khalf = lane >> 5;
    const int img = __builtin_amdgcn_readfirstlane(n);
    const int rows0 = __builtin_amdgcn_readfirstlane(i_base);
    const int image_bytes = p.Co * p.HoWo * 2;
    const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc(
        (uint16_t*)p.out + (size_t)img * p.out_ns, (short)0, image_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_mask = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>((const uint16_t*)(has_mask ? p.mask : p.out)) + (size_t)img * p.out_ns, (short)0, image_bytes, 0x00020000);
    // lanes past the tile's last pixel: an offset outside every resource
    const unsigned voff = pix_first < pix_end ? (unsigned)(pix_first + khalf * 4 * p.HoWo) * 2u : 0x80000000u;
    auto load_packet = [&](const __amdgpu_buffer_rsrc_t& r, int soff) {
        packet_t v;
        if constexpr (TN == 2) v[0] = __builtin_amdgcn_raw_buffer_load_b32(r, voff, soff, 0);
        else v = __builtin_amdgcn_raw_buffer_load_b64(r, voff, soff, 0);
        return v;
    };
    auto rows = [&](auto relu_c) {
        constexpr bool RELU = decltype(relu_c)::value;
#pragma unroll
        for (int a = 0; a < TM; ++a) {
            // the bias of an accumulator quad's four consecutive rows as one 16-byte LDS read, all four
            // quads requested before the first is used
            floatx4 bq[4];
            if (FUSED && FWD) {
#pragma unroll
                for (int qd = 0; qd < 4; ++qd) {
                    const floatx4 z = {0.0f, 0.0f, 0.0f, 0.0f};
                    bq[qd] = has_bias ? *reinterpret_cast<const floatx4*>(&bias_lds[i_base + a * 32 + qd * 8 + khalf * 4 - i_tile0]) : z;
                }
            }
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int soff = (rows0 + a * 32 + (e >> 2) * 8 + (e & 3)) * p.HoWo * 2;   // scalar: the lane's khalf * 4 rows sit in voff
                float x[TN];
#pragma unroll
                for (int b = 0; b < TN; ++b) x[b] = acc[a][b][e];
                if (FUSED && FWD) {
#pragma unroll
                    for (int b = 0; b < TN; ++b) x[b] += bq[e >> 2][e & 3];
                }
                if (RELU) {
#pragma unroll
                    for (int b = 0; b < TN; ++b) x[b] = x[b] > 0.0f ? x[b] : 0.0f;
                }
                if (has_mask) {
                    const packet_t m = load_packet(r_mask, soff);
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        const uint32_t w = m[b >> 1];
                        x[b] = __uint_as_float((b & 1) ? (w & 0xffff0000u) : (w << 16)) > 0.0f ? x[b] : 0.0f;
                    }
                }
                if (has_beta) {
                    const packet_t o = load_packet(r_out, soff);
#pragma unroll
                    for (int b = 0; b < TN; ++b) {
                        const uint32_t w = o[b >> 1];
                        x[b] += __uint_as_float((b & 1) ? (w & 0xffff0000u) : (w << 16));
                    }
                }
                packet_t r;
#pragma unroll
                for (int b = 0; b < TN; b += 2) r[b >> 1] = pack_bf16(x[b], x[b + 1]);
                if constexpr (TN == 2) __builtin_amdgcn_raw_buffer_store_b32(r[0], r_out, voff, soff, 0);
                else __builtin_amdgcn_raw_buffer_store_b64(r, r_out, voff, soff, 0);
            }
        }
    };
    if (relu) rows(std::true_type{}); else rows(std::false_type{});
}

// Depth-to-space epilogue of stride-2 x stride-2 phase-folded backward-data for kernels whose lanes
// own TN coarse pixels (hq_of[b], wq_of[b]) of ONE image (bf16 dx, NCHW). Row i of the tile is (c, a, b) =
// (i / 4, (i / 2) % 2, i % 2) and lands at dx[n, c, hq*2 + a - ph, wq*2 + b - pw]. For accumulator
// register e of a lane, a and b depend on e alone and c is a scalar plus the lane's half, so a lane
// needs, per coarse pixel, the four offsets of its (a, b) positions (outside the image: an offset
// outside the resource), and a store is a conversion and one raw buffer store with a scalar channel
// offset; channels at or past C fall outside the resource, which covers image n. (The general
// depth-to-space epilogue decodes every element's row with reciprocal divisions and tests its
// position, some forty instructions per 2-byte store.)
template <bool FUSED, int TM, int TN>
__device__ __forceinline__ void store_d2s2_adjacent(const PixParams& p, floatx16 (&acc)[TM][TN], int i_base, int n,
                                                    const int (&hq_of)[TN], const int (&wq_of)[TN], const bool (&live_of)[TN],
                                                    int lane) {
    const bool has_mask = FUSED && p.mask != nullptr, has_beta = p.beta != 0.0f;
    const int khalf = lane >> 5;
    const int img = __builtin_amdgcn_readfirstlane(n);
    const int rows0 = __builtin_amdgcn_readfirstlane(i_base);
    const int plane = p.H * p.W;
    const int image_bytes = p.C * plane * 2;
    const __amdgpu_buffer_rsrc_t r_out = __builtin_amdgcn_make_buffer_rsrc(
        (uint16_t*)p.out + (size_t)img * p.out_ns, (short)0, image_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t r_mask = __builtin_amdgcn_make_buffer_rsrc(
        const_cast<uint16_t*>((const uint16_t*)(has_mask ? p.mask : p.out)) + (size_t)img * p.out_ns, (short)0, image_bytes, 0x00020000);
    unsigned voff[TN][2][2];
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const bool live = live_of[b];
        const int hb = (hq_of[b] + p.hq_min) * 2 - p.ph, wb = (wq_of[b] + p.wq_min) * 2 - p.pw;
#pragma unroll
        for (int pa = 0; pa < 2; ++pa)
#pragma unroll
            for (int pb = 0; pb < 2; ++pb) {
                const int h = hb + pa, w = wb + pb;
                const bool ok = live & ((unsigned)h < (unsigned)p.H) & ((unsigned)w < (unsigned)p.W);
                voff[b][pa][pb] = ok ? (unsigned)(khalf * plane + h * p.W + w) * 2u : 0x80000000u;
            }
    }
#pragma unroll
    for (int a = 0; a < TM; ++a) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            // row = rows0 + a*32 + (e>>2)*8 + khalf*4 + (e&3): channel (rows0 + a*32 + (e>>2)*8) / 4 + khalf, phase (e&3)
            const int c_lo = (rows0 + a * 32 + (e >> 2) * 8) >> 2;      // scalar
            if (c_lo >= p.C) continue;                                    // uniform: both halves past the last channel
            const int soff = c_lo * plane * 2;
            constexpr int dummy = 0; (void)dummy;
            const int pa = (e & 3) >> 1, pb = e & 1;
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const unsigned vo = voff[b][pa][pb];
                float v = acc[a][b][e];
                if (has_mask)
                    v = __uint_as_float((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r_mask, vo, soff, 0) << 16) > 0.0f ? v : 0.0f;
                if (has_beta) v += __uint_as_float((uint32_t)__builtin_amdgcn_raw_buffer_load_b16(r_out, vo, soff, 0) << 16);
                __builtin_amdgcn_raw_buffer_store_b16((uint16_t)(pack_bf16(v, 0.0f) & 0xffffu), r_out, vo, soff, 0);
            }
        }
    }
}

// Consecutive workgroup ids land on different XCDs (8 per chip, each with its own L2). Give each
// XCD a contiguous run of tiles so that neighbouring pixel tiles share halo rows in one L2.
__device__ __forceinline__ int xcd_tile(int bid, int total) {
    const int per = total >> 3;
    return (per > 0 && bid < per * 8) ? (bid & 7) * per + (bid >> 3) : bid;
}


struct TileCfg { int bm, bn; float eff; };

// (TM, TN, WM, WN) for each tile extent: workgroup = WM x WN wavefronts of TM x TN MFMA tiles (32x32)
#define PURINE_TILE_SWITCH(CALL)                                       \
    switch (bm * 1000 + bn) {                                          \
        case 192128: return CALL(3, 2, 2, 2);                          \
        case 128128: return CALL(2, 2, 2, 2);                          \
        case 96256:  return CALL(3, 2, 1, 4);                          \
        case 96128:  return CALL(3, 1, 1, 4);                          \
        case 64256:  return CALL(2, 2, 1, 4);                          \
        case 128064: return CALL(1, 2, 4, 1);                          \
        case 64128:  return CALL(2, 1, 1, 4);                          \
        case 32256:  return CALL(1, 2, 1, 4);                          \
        case 64064:  return CALL(1, 1, 2, 2);                          \
        case 32128:  return CALL(1, 1, 1, 4);                          \
        default: return hipErrorInvalidValue;                          \
    }

// bf16 MFMA variant of the tap kernel (conv_igemm_bf16.hip). mode: 0 fwd, 1 bwd unit stride, 2 bwd phase-folded.
hipError_t dispatch_tap_bf16(PixParams& p, int mode, int bm, int bn, hipStream_t st);
// bf16 tap kernels gather from a channels-blocked copy [N][Ci_pad/8][Hi][Wi][8] of p.in: this writes
// it into `blocked` (N*Ci_pad*Hi*Wi*2 bytes, 16-byte aligned) and points p.in at it
hipError_t blockify_input(PixParams& p, void* blocked, hipStream_t st);
// single-tap bf16 layers (mode 0 or 1): no blocked copy, 2-byte gathers from NCHW
hipError_t dispatch_tap_bf16_nchw(PixParams& p, int mode, int bm, int bn, hipStream_t st);
// bf16 layers whose gather has unit stride and whose gathered rows are whole 16-byte packets: the
// haloed input patch of a pixel tile is staged in LDS once per 16-channel group and every tap
// reads it there (conv_patch_bf16.hip). plan_patch_bf16 answers whether the layer qualifies (pure
// host arithmetic on p's geometry) and, if so, sets p.Ci_pad / p.i_pad / p.tiles_i / p.tiles_pix /
// p.in_bytes for the tile it picked; the caller then repacks the filter into scratch of at least
// patch_filter_bytes (repack_patch_filter) and launches.
// mode: 0 forward, 1 backward-data with unit stride, 2 backward-data phase-folded.
struct PatchGeom {
    int bm, bn, rounds;  // tile extents; patch fill tasks per thread and channel group
    int tiles_per_img;   // pixel tiles per image (a tile never straddles two images)
    int pw;              // patch columns: Wo + St - 1
    int pr_max;          // patch rows held in LDS
    int w_lo;            // input column of patch column 0 (<= 0)
    int h_lo_add;        // input row of patch row 0 = first output row of the tile + h_lo_add
    int pos_add;         // backward walk: (Rt-1)*pw + (St-1), else 0
    int chunks;          // 16-byte packets per input row: Wi / 8
    int halo_l, halo_r0; // patch columns [0, halo_l) and [halo_r0, pw) lie outside the image
    int taps_per_stage;  // taps whose filter rows sit in LDS together
    int a_rounds;        // 16-byte filter pieces per thread and stage
    int pairs;           // NCHW output written as 4-byte pixel pairs
    int a_bytes, lds_bytes;
    int plane_bytes;     // bytes of one (position parity, channel half) plane of the patch
    int tasks_per_row;   // fill tasks per patch row: packets rounded up to fours x two halves
    int d2s_buffers;     // phase-folded backward-data: the depth-to-space epilogue may use raw buffer stores
    int roles;           // 1: the persistent kernel whose wavefronts split into fill and multiply roles
    int roles_lds;       // its LDS bytes
    int wv;              // ... and the row width its pixel tiles count in: Wo rounded up to whole groups of four
    FastDiv div_wv;
    FastDiv div_tpi, div_tpr, div_chunks, div_halo, div_st;
};
bool plan_patch_bf16(PixParams& p, int mode, PatchGeom* q);
size_t patch_filter_bytes(int Co, int Ci, int n_taps);
hipError_t repack_patch_filter(const PixParams& p, int mode, const void* w, void* a, int K, int C, hipStream_t st);
hipError_t launch_patch_bf16(const PixParams& p, const PatchGeom& q, int mode, hipStream_t st);
// bf16 forward for layers with fewer than 16 input channels whose input rows are whole 16-byte
// packets (conv_rows_bf16.hip): input rows staged in LDS in their natural layout, the reduction runs
// over (c, r, block of 8 filter columns), persistent workgroups. plan_rows_bf16 answers whether the
// layer qualifies and fills q (and p.tiles_i / p.i_pad / p.in_bytes); launch_rows_bf16 repacks the
// filter into ws (rows_filter_bytes) and launches.
struct RowsGeom {
    int SB, n_blocks, n_steps;   // blocks of 8 filter columns per filter row; (c, r, block) count; MFMA steps (2 blocks each)
    int origin, rowlen;          // element of an LDS row that holds input column 0; elements per LDS row
    int pr_max;                  // input rows per channel held for one pixel tile
    int chunks, fill_rounds;     // 16-byte packets per input row; packets per thread and tile
    int a_pitch, lds_bytes;
    int tiles_per_img, n_tiles, grid, pairs;
    FastDiv div_tpi, div_chunks, div_pr;
};
bool plan_rows_bf16(PixParams& p, RowsGeom* q);
size_t rows_filter_bytes(int K, int C, int R, int S);
hipError_t launch_rows_bf16(const PixParams& p, const RowsGeom& q, const void* w, void* ws, hipStream_t st);
// bf16 MFMA forward with a flattened (c,r,s) reduction (fewer than 16 input channels)
hipError_t dispatch_flat_bf16(PixParams& p, int bm, int bn, hipStream_t st);
// streaming GEMM for 1x1 / stride 1 / unpadded layers (conv_gemm1x1.hip); p.wt is the KCRS filter
hipError_t dispatch_gemm1x1(const PixParams& p, int dtype, bool trans, int tm, int tn, hipStream_t st);

}  // namespace pix
}  // namespace purine

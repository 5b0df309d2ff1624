// bf16 MFMA forward convolution for layers with few input channels (the first layer of a CNN:
// Conv of paper Figure 1(b) with C < 16), any stride.
//
// The reduction index is (c, r, block of 8 filter columns): the 8 consecutive filter columns of one
// filter row multiply 8 consecutive input columns, which are contiguous in NCHW, so a lane's MFMA
// operand (8 consecutive reduction elements) is one 16-byte window of an input row. A workgroup
// stages the input rows its pixel tile touches in LDS in their NATURAL layout (16-byte packets
// straight from global memory, no transposition, zero halo on both sides) and every (c, r, block)
// reads its windows there: window start = stride * wo - pad + 8 * block, 4-byte aligned dword reads
// plus a funnel shift when the start is an odd element. The filter, repacked once to
// A[k][(c, r, block)][8] with zeros in the columns past S, stays in LDS for the whole kernel:
// workgroups are persistent and walk over pixel tiles with a double-buffered row patch, one barrier
// per tile (the next tile's rows are loaded during the current tile's MFMAs).
#include "pix_common.h"

namespace purine {
namespace pix {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int FILL_ROUNDS = 6;   // 16-byte packets per thread and tile, at most

template <bool FUSED, int TM, int TN, int WM, int WN>
__global__ __launch_bounds__(256, 2) void conv_rows_bf16_kernel(const PixParams p, const RowsGeom q) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    static_assert(NT == 256, "four wavefronts");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* bias_s = reinterpret_cast<float*>(smem);                 // [BM]
    unsigned char* As = smem + BM * 4;                              // [BM] rows of a_pitch bytes
    unsigned char* rows = As + BM * q.a_pitch;                      // [2][C * pr_max] rows of rowlen elements

    const uint16_t* __restrict__ in = (const uint16_t*)p.in;
    const uint16_t* __restrict__ wt = (const uint16_t*)p.wt;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;
    const int khalf = lane >> 5;

    const int i0 = (blockIdx.x % p.tiles_i) * BM;
    const int worker = blockIdx.x / p.tiles_i, n_workers = gridDim.x / p.tiles_i;
    const int buf_bytes = p.C * q.pr_max * q.rowlen * 2;

    // ---- once: the filter rows of this row tile, the bias, zeros in both halos of both row buffers
    for (int f = tid; f < BM * q.n_steps * 2; f += NT) {
        const int row = f / (q.n_steps * 2), piece = f - row * (q.n_steps * 2);
        u32x4 v = {0u, 0u, 0u, 0u};
        if (i0 + row < p.Co) v = *reinterpret_cast<const u32x4*>(wt + ((size_t)(i0 + row) * q.n_steps * 2 + piece) * 8);
        *reinterpret_cast<u32x4*>(As + row * q.a_pitch + piece * 16) = v;
    }
    if (FUSED) stage_bias<uint16_t, BM, NT>(bias_s, p, i0, tid);
    {
        const int right = (q.rowlen - q.origin - p.W) / 8;          // 16-byte pieces right of the image
        const int per_row = q.origin / 8 + right;
        const int total = 2 * p.C * q.pr_max * per_row;
        for (int i = tid; i < total; i += NT) {
            const int row = i / per_row, piece = i - row * per_row;
            const int el = piece < q.origin / 8 ? piece * 8 : q.origin + p.W + (piece - q.origin / 8) * 8;
            const u32x4 z = {0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4*>(rows + (row * q.rowlen + el) * 2) = z;
        }
    }

    // ---- fill tasks of this thread: (channel, patch row, packet), fixed; the image and first row change per tile
    int f_goff[FILL_ROUNDS], f_pr[FILL_ROUNDS], f_lds[FILL_ROUNDS];
    const int tasks = p.C * q.pr_max * q.chunks;
#pragma unroll
    for (int r = 0; r < FILL_ROUNDS; ++r) {
        const int t = tid + r * NT;
        const int row = fastdiv(t, q.div_chunks);
        const int chunk = t - row * q.chunks;
        const int c = fastdiv(row, q.div_pr);
        const int pr = row - c * q.pr_max;
        const bool live = t < tasks;
        f_goff[r] = (c * p.H * p.W + chunk * 8) * 2;
        f_pr[r] = live ? pr : -0x40000000;                          // a dead task always reads "outside the image"
        f_lds[r] = live ? (row * q.rowlen + q.origin + chunk * 8) * 2 : -1;
    }
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(in), (short)0, (int)p.in_bytes, 0x00020000);
    u32x4 pre[FILL_ROUNDS];
    auto load_rows = [&](int tile) {
        const int n = fastdiv(tile, q.div_tpi);
        const int pix0 = (tile - n * q.tiles_per_img) * BN;
        const int h0 = fastdiv(pix0, p.div_wo) * p.sh - p.ph;       // input row of patch row 0
        const int img = n * p.in_ns * 2;
#pragma unroll
        for (int r = 0; r < FILL_ROUNDS; ++r) {
            if (r >= q.fill_rounds) break;                          // uniform
            const int hi = h0 + f_pr[r];
            const unsigned v = (unsigned)hi < (unsigned)p.H ? (unsigned)(img + f_goff[r] + hi * p.W * 2) : 0x80000000u;
            pre[r] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, v, 0, 0);
        }
    };
    auto store_rows = [&](int buf) {
#pragma unroll
        for (int r = 0; r < FILL_ROUNDS; ++r) {
            if (r >= q.fill_rounds) break;
            if (f_lds[r] >= 0) *reinterpret_cast<u32x4*>(rows + buf * buf_bytes + f_lds[r]) = pre[r];
        }
    };

    const int a_row = (wm * TM * 32 + (lane & 31)) * q.a_pitch + khalf * 16;

    // A worker takes a contiguous range of pixel tiles: consecutive tiles of an image share most of
    // their input rows, and the rows a tile loads again were fetched a tile ago by the same workgroup
    // (tiles dealt out round-robin put neighbours on different XCDs, each fetching the shared rows
    // into its own L2: the counters showed the input read 2.9 times from memory).
    const int per_worker = (q.n_tiles + n_workers - 1) / n_workers;
    int tile = worker * per_worker;
    const int tile_end = min(tile + per_worker, q.n_tiles);
    if (tile < tile_end) load_rows(tile);
    store_rows(0);
    __syncthreads();

    int buf = 0;
    for (; tile < tile_end; ++tile) {
        const int n = fastdiv(tile, q.div_tpi);
        const int pix0 = (tile - n * q.tiles_per_img) * BN;
        const int pix_end = min(pix0 + BN, p.HoWo);
        const int ho_first = fastdiv(pix0, p.div_wo);
        const int next = tile + 1;
        if (next < tile_end) load_rows(next);                       // lands during this tile's MFMAs

        // this lane's window origin (element index inside the buffer) for tap row 0, block 0 of channel 0
        int b_el[TN];
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int pix = min(pix0 + wn * TN * 32 + TN * (lane & 31) + b, pix_end - 1);   // a lane's tiles: adjacent pixels
            const int ho = fastdiv(pix, p.div_wo);
            const int wo = pix - ho * p.Wo;
            b_el[b] = (ho - ho_first) * p.sh * q.rowlen + wo * p.sw + q.origin - p.pw;
        }
        floatx16 acc[TM][TN];
#pragma unroll
        for (int a = 0; a < TM; ++a)
#pragma unroll
            for (int b = 0; b < TN; ++b)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

        const unsigned char* cur = rows + buf * buf_bytes;
        // this lane's reduction block (c, r, sb) = 2 * step + khalf, walked in registers (mixed radix
        // SB, R): no table look-up stands between a step and its window reads
        int k_sb = khalf % q.SB, k_r = khalf / q.SB, k_c = 0;
        if (k_r >= p.R) { k_r -= p.R; k_c = 1; }
        for (int t = 0; t < q.n_steps; ++t) {
            // the padding block past the last real one multiplies zero weights: it re-reads block 0
            const int blk = k_c < p.C ? (k_c * q.pr_max + k_r) * q.rowlen + k_sb * 8 : 0;
            bf16x8 av[TM], bv[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a)
                av[a] = *reinterpret_cast<const bf16x8*>(As + a_row + a * 32 * q.a_pitch + t * 32);
#pragma unroll
            for (int b = 0; b < TN; ++b) {
                const int el = b_el[b] + blk;
                const uint32_t* src = reinterpret_cast<const uint32_t*>(cur + (el & ~1) * 2);
                const uint32_t d0 = src[0], d1 = src[1], d2 = src[2], d3 = src[3], d4 = src[4];
                const unsigned shift = (el & 1) * 16;               // odd start: drop the first half-dword
                u32x4 w;
                w[0] = __builtin_amdgcn_alignbit(d1, d0, shift);
                w[1] = __builtin_amdgcn_alignbit(d2, d1, shift);
                w[2] = __builtin_amdgcn_alignbit(d3, d2, shift);
                w[3] = __builtin_amdgcn_alignbit(d4, d3, shift);
                bv[b] = __builtin_bit_cast(bf16x8, w);
            }
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[a], bv[b], acc[a][b], 0, 0, 0);
            // two blocks on
            k_sb += 2;
            const int c1 = k_sb >= 2 * q.SB ? 2 : (k_sb >= q.SB ? 1 : 0);
            k_sb -= c1 * q.SB;
            k_r += c1;
            const int c2 = k_r >= 2 * p.R ? 2 : (k_r >= p.R ? 1 : 0);
            k_r -= c2 * p.R;
            k_c += c2;
        }

        store_rows(buf ^ 1);                                        // nobody reads that buffer during this tile
        if (q.pairs)
            store_adjacent<FUSED, TM, TN, true>(p, acc, i0 + wm * TM * 32, n, pix0 + wn * TN * 32 + TN * (lane & 31),
                                                pix_end, lane, bias_s, i0);
        else
            store_tile<uint16_t, false, FUSED, TM, TN, true>(p, (uint16_t*)p.out, acc, i0 + wm * TM * 32,
                                                             n * p.HoWo + pix0 + wn * TN * 32 + TN * (lane & 31), khalf,
                                                             bias_s, i0, n * p.HoWo + pix_end, 1);
        __syncthreads();
        buf ^= 1;
    }
}

// A[k_pad][n_steps * 2 blocks][8]: block (c, r, sb) holds w[k][c][r][8*sb .. 8*sb+7], zero past S and
// past the last block / row.
struct RowsRepack {
    const uint16_t* w; uint16_t* a;
    int K, C, R, S, SB, n_blocks, n_steps, k_pad, total;
};
__global__ __launch_bounds__(256) void repack_rows_kernel(const RowsRepack g) {
    for (int o = blockIdx.x * 256 + threadIdx.x; o < g.total; o += gridDim.x * 256) {
        const int e = o & 7;
        int t = o >> 3;
        const int blk = t % (g.n_steps * 2);
        const int k = t / (g.n_steps * 2);
        uint16_t v = 0;
        if (k < g.K && blk < g.n_blocks) {
            const int sb = blk % g.SB;
            const int cr = blk / g.SB;
            const int r = cr % g.R, c = cr / g.R;
            const int s = sb * 8 + e;
            if (s < g.S) v = g.w[((k * g.C + c) * g.R + r) * g.S + s];
        }
        g.a[o] = v;
    }
}

template <bool FUSED>
hipError_t launch_rows(const PixParams& p, const RowsGeom& q, hipStream_t st) {
    auto kern = conv_rows_bf16_kernel<FUSED, 2, 2, 1, 4>;          // 64 rows x 256 pixels
    if (q.lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, q.lds_bytes);
        if (e != hipSuccess) return e;
    }
    ProbeScope probe(st);
    (void)hipGetLastError();
    hipLaunchKernelGGL(kern, dim3((unsigned)q.grid), dim3(256), (size_t)q.lds_bytes, st, p, q);
    return hipGetLastError();
}

}  // namespace

// p: forward geometry as the flattened kernel gets it. On success p.tiles_i / p.i_pad / p.in_bytes
// and q describe this kernel's launch.
bool plan_rows_bf16(PixParams& p, RowsGeom* qg) {
    constexpr int BM = 64, BN = 256;
    if ((p.W & 7) || (p.in_ns & 7) || p.pw > 7 || p.ph < 0) return false;
    if ((((uintptr_t)p.in) & 15u) != 0) return false;
    const long long in_bytes = ((long long)(p.N - 1) * p.in_ns + (long long)p.C * p.H * p.W) * 2;
    if (in_bytes >= 0x7fffffffLL) return false;
    RowsGeom q{};
    q.SB = (p.S + 7) / 8;
    q.n_blocks = p.C * p.R * q.SB;
    q.n_steps = (q.n_blocks + 1) / 2;
    q.origin = 8;
    // furthest element a window read touches: last pixel of a row, last block, 10 elements (5 dwords)
    const int reach = q.origin - p.pw + p.sw * (p.Wo - 1) + 8 * (q.SB - 1) + 10;
    int rowlen = q.origin + p.W + 8;
    if (reach > rowlen) rowlen = reach;
    q.rowlen = (rowlen + 7) / 8 * 8;
    const int rows_spanned = (BN - 2) / p.Wo + 2;
    q.pr_max = p.sh * ((rows_spanned < p.Ho ? rows_spanned : p.Ho) - 1) + p.R;
    q.chunks = p.W / 8;
    const long long tasks = (long long)p.C * q.pr_max * q.chunks;
    if (tasks > FILL_ROUNDS * 256) return false;
    q.fill_rounds = (int)((tasks + 255) / 256);
    q.a_pitch = q.n_steps * 32 + 16;
    const long long lds = (long long)BM * 4 + (long long)BM * q.a_pitch + 2ll * p.C * q.pr_max * q.rowlen * 2;
    if (lds > 80 * 1024) return false;
    q.lds_bytes = (int)lds;
    q.tiles_per_img = (p.HoWo + BN - 1) / BN;
    const long long n_tiles = (long long)p.N * q.tiles_per_img;
    if (n_tiles > 0x7fffffffLL) return false;
    q.n_tiles = (int)n_tiles;
    p.tiles_i = (p.Co + BM - 1) / BM;
    p.i_pad = p.tiles_i * BM;
    long long workers = 512 / p.tiles_i;                            // two workgroups per CU in all
    if (workers < 1) workers = 1;
    if (workers > n_tiles) workers = n_tiles;
    q.grid = (int)(workers * p.tiles_i);
    q.div_tpi = make_fastdiv(q.tiles_per_img);
    q.div_chunks = make_fastdiv(q.chunks);
    q.div_pr = make_fastdiv(q.pr_max);
    // TN = 2 adjacent pixels per lane; that epilogue addresses one image of the output as a raw buffer
    q.pairs = ((p.HoWo | p.out_ns) & 1) == 0 && (((uintptr_t)p.out) & 3u) == 0 && (long long)p.Co * p.HoWo * 2 < 0x7fffffffLL;
    p.in_bytes = (unsigned)in_bytes;
    *qg = q;
    return true;
}

size_t rows_filter_bytes(int K, int C, int R, int S) {
    const long long blocks = ((long long)C * R * ((S + 7) / 8) + 1) / 2 * 2;
    return (size_t)((K + 63) / 64 * 64) * (size_t)blocks * 16;
}

hipError_t launch_rows_bf16(const PixParams& p, const RowsGeom& q, const void* w, void* ws, hipStream_t st) {
    RowsRepack g{};
    g.w = (const uint16_t*)w; g.a = (uint16_t*)ws;
    g.K = p.Co; g.C = p.C; g.R = p.R; g.S = p.S; g.SB = q.SB; g.n_blocks = q.n_blocks; g.n_steps = q.n_steps;
    g.k_pad = p.i_pad;
    g.total = p.i_pad * q.n_steps * 16;
    const int blocks = (g.total + 255) / 256;
    (void)hipGetLastError();
    hipLaunchKernelGGL(repack_rows_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(256), 0, st, g);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    PixParams pp = p;
    pp.wt = ws;
    const bool fused = p.bias || p.relu;
    return fused ? launch_rows<true>(pp, q, st) : launch_rows<false>(pp, q, st);
}

}  // namespace pix
}  // namespace purine

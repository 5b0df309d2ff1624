// bf16 weight gradient for 3x3 / stride 1 / pad 1 layers with rows of whole 16-byte packets
// (ConvBwdWeight of paper Figure 1(b)):
//
//     dw[k, c, r, s] = sum over (n, p, q) of dy[n, k, p, q] * x[n, c, p - 1 + r, q - 1 + s]
//
// The reduction runs over pixels, and NCHW keeps the pixels of a row contiguous, so BOTH MFMA
// operands (8 consecutive reduction elements per lane) are 16-byte windows of rows as they lie in
// memory: dy[k][p][q0..q0+7] and x[c][p-1+r][q0-1+s .. q0+6+s]. A workgroup walks over output rows;
// per row it holds in LDS, in their natural layout, the dy row of its 64 output channels and a ring
// of the input rows of its 64 input channels (consecutive output rows share two of their three
// input rows, so each step brings in ONE new input row and one dy row, 16-byte packets straight
// from global memory). The three column taps of a filter row read the same aligned packet plus the
// dword on either side, taken from the partner lane's registers, and are shifted into place in
// registers (funnel shifts), so a step of 16 pixels costs a wavefront 4 LDS reads for 9 MFMAs. Each wavefront owns 32 output channels x 32
// input channels x all nine taps (144 accumulators). Workgroups are persistent over a contiguous
// range of (image, row) pairs; their fp32 partial tiles go to scratch as [split][tap][k][c] and the
// fixed-order second pass of the general kernel adds them.
#include "common.h"

namespace purine {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64, CT = 64;     // output / input channels per workgroup
constexpr int ORG = 8;              // element of an x row in LDS that holds image column 0
constexpr int LOADS = 2;            // 16-byte packets per thread and step, at most, per operand (rows of up to 64 pixels)

// LDS row pitch: at least `bytes`, and 16 bytes past a multiple of 128, so that the 16-byte reads of 8
// consecutive rows (lanes run along channels) fall into distinct bank groups
inline int row_pitch(int bytes) { return (bytes - 16 + 127) / 128 * 128 + 16; }

struct RowsWgradParams {
    const uint16_t* x; const uint16_t* dy; float* out; float* db_out;
    int N, C, H, W, K, P, Q;
    int x_ns, dy_ns;
    unsigned x_bytes, dy_bytes;
    int k_groups, c_groups, workers;   // grid = k_groups * c_groups * workers
    int rows_total, rows_per_worker;   // flattened (n, p) output rows
    int xpitch, dypitch;               // LDS bytes per x row / dy row
    int xchunks, dychunks;             // 16-byte packets per x row (W / 8) and dy row (Q / 8)
    int steps;                         // 16-pixel MFMA steps per output row: ceil(Q / 16)
    int x_rounds, d_rounds;            // 16-byte packets per thread and step for each operand
    FastDiv div_p, div_xchunks, div_dychunks;
};

__device__ __forceinline__ float sum8(const u32x4 u) {
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += __uint_as_float(u[i] << 16) + __uint_as_float(u[i] & 0xffff0000u);
    return s;
}

__global__ __launch_bounds__(256, 2) void wgrad_rows3x3_bf16_kernel(const RowsWgradParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* xs = smem;                                   // [4 ring slots][CT] rows of xpitch bytes
    unsigned char* dys = smem + 4 * CT * p.xpitch;              // [2][KT] rows of dypitch bytes

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int khalf = lane >> 5;
    const int wk = wave >> 1, wc = wave & 1;                    // this wavefront's 32-row k tile and 32-channel tile

    // blockIdx -> (worker, k group, c group): the groups of one worker read the same rows, so they
    // share an XCD (consecutive ids go round the 8 XCDs)
    const int per_worker = p.k_groups * p.c_groups;
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int worker = (j / per_worker) * 8 + xcd;
    const int grp = j % per_worker;
    const int k0 = (grp / p.c_groups) * KT, c0 = (grp % p.c_groups) * CT;

    const int g0 = worker * p.rows_per_worker;
    const int g1 = min(g0 + p.rows_per_worker, p.rows_total);

    // ---- once: zero everything (halos of the x rows, the tail of the dy rows)
    {
        const int total = (4 * CT * p.xpitch + 2 * KT * p.dypitch) / 16;
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < total; i += 256) *reinterpret_cast<u32x4*>(smem + i * 16) = z;
    }

    // ---- load tasks of this thread (fixed): x packets (channel, packet) and dy packets (k, packet)
    int x_goff[LOADS], x_lds[LOADS], d_goff[LOADS], d_lds[LOADS];
    const int x_tasks = CT * p.xchunks, d_tasks = KT * p.dychunks;
#pragma unroll
    for (int r = 0; r < LOADS; ++r) {
        const int t = tid + r * 256;
        const int c = fastdiv(t, p.div_xchunks), ch = t - c * p.xchunks;
        const bool xl = t < x_tasks && c0 + c < p.C;
        x_goff[r] = xl ? ((c0 + c) * p.H * p.W + ch * 8) * 2 : -1;
        x_lds[r] = t < x_tasks ? c * p.xpitch + (ORG + ch * 8) * 2 : -1;
        const int k = fastdiv(t, p.div_dychunks), dch = t - k * p.dychunks;
        const bool dl = t < d_tasks && k0 + k < p.K;
        d_goff[r] = dl ? ((k0 + k) * p.P * p.Q + dch * 8) * 2 : -1;
        d_lds[r] = t < d_tasks ? k * p.dypitch + dch * 16 : -1;
    }
    const __amdgpu_buffer_rsrc_t rs_x =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.x), (short)0, (int)p.x_bytes, 0x00020000);
    const __amdgpu_buffer_rsrc_t rs_dy =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(p.dy), (short)0, (int)p.dy_bytes, 0x00020000);
    u32x4 xr[LOADS], dr[LOADS];
    // input row h of image n (zeros when outside the image) and dy row (n, pp) (zeros unless `real`)
    auto load_step = [&](int n, int h, bool real_dy, int pp) {
        const bool x_ok = (unsigned)h < (unsigned)p.H;
        const int xb = n * p.x_ns * 2 + h * p.W * 2;
        const int db = n * p.dy_ns * 2 + pp * p.Q * 2;
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            if (r >= p.x_rounds) break;          // uniform
            const unsigned vx = (x_ok && x_goff[r] >= 0) ? (unsigned)(xb + x_goff[r]) : 0x80000000u;
            xr[r] = __builtin_amdgcn_raw_buffer_load_b128(rs_x, vx, 0, 0);
        }
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            if (r >= p.d_rounds) break;
            const unsigned vd = (real_dy && d_goff[r] >= 0) ? (unsigned)(db + d_goff[r]) : 0x80000000u;
            dr[r] = __builtin_amdgcn_raw_buffer_load_b128(rs_dy, vd, 0, 0);
        }
    };
    auto store_step = [&](int slot, int dbuf) {
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            if (r >= p.x_rounds) break;
            if (x_lds[r] >= 0) *reinterpret_cast<u32x4*>(xs + slot * CT * p.xpitch + x_lds[r]) = xr[r];
        }
#pragma unroll
        for (int r = 0; r < LOADS; ++r) {
            if (r >= p.d_rounds) break;
            if (d_lds[r] >= 0) *reinterpret_cast<u32x4*>(dys + dbuf * KT * p.dypitch + d_lds[r]) = dr[r];
        }
    };

    floatx16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;
    float dbacc = 0.0f;
    const bool do_db = p.db_out != nullptr && c0 == 0 && wc == 0;

    if (g0 < g1) {
        // Extended row index pe of an image runs from -1 to P + 1: step pe loads input row pe into ring
        // slot pe & 3 and the dy row of step pe + 1, and multiplies output row pe - 2 (when that row
        // exists and belongs to this worker) with input rows pe - 3 .. pe - 1. The first three steps of
        // a range only fill the ring.
        int n = fastdiv(g0, p.div_p);
        int pe = g0 - n * p.P - 1;          // first step: loads row p0 - 1
        int g = g0 - 3;                      // flattened output row this step multiplies (pe - 2 of image n)
        __syncthreads();                     // zeros in place
        // step "pe - 1" of the walk: nothing in flight yet, so load the first row here
        load_step(n, pe, false, 0);
        store_step(pe & 3, 0);
        __syncthreads();
        pe += 1; g += 1;
        int dbuf = 0;                        // dy buffer the CURRENT step reads
        while (true) {
            // next step's operands: input row pe, dy row of output row (pe + 1) - 2 = pe - 1
            const bool next_real = pe - 1 >= 0 && pe - 1 < p.P && g + 1 >= g0 && g + 1 < g1;
            load_step(n, pe, next_real, pe - 1);
            const bool real = pe - 2 >= 0 && pe - 2 < p.P && g >= g0;
            if (real) {
                const unsigned char* a_base = dys + dbuf * KT * p.dypitch + (wk * 32 + (lane & 31)) * p.dypitch + khalf * 16;
                const int xrow = (wc * 32 + (lane & 31)) * p.xpitch + (ORG + khalf * 8) * 2;   // column 8h of the lane's channel
                const unsigned char* rowp[3];
#pragma unroll
                for (int r = 0; r < 3; ++r) rowp[r] = xs + ((pe - 3 + r) & 3) * CT * p.xpitch + xrow;
                // Column taps by shifting dy, not x: with q' = q - 1 + s the sum over q of
                // dy[q] * x[q - 1 + s] is the sum over the real columns q' of dy[q' + 1 - s] * x[q'] (the
                // padding columns of x contribute nothing). The three input rows' packets then serve all
                // three column taps as they are, and only the one dy fragment is shifted, by one pixel
                // either way (funnel shifts). The dword next to a lane's dy packet is the last / first
                // dword of its partner lane's packet (the other 8-pixel half of the same channel): the
                // same step's for the inner side of the pair, the previous / next step's for the outer
                // side. So the MFMAs of tap s = 0 (dy one pixel to the right) are issued one step late,
                // when the next step's packet is in registers, and no dword is fetched from LDS on its
                // own (4-byte reads at this row pitch fall on 8 banks: each cost as much as a 16-byte
                // one). Every accumulator still takes its steps in ascending order.
                u32x4 pav = {0u, 0u, 0u, 0u}, pd[3];       // previous step: dy fragment, x packets
#pragma unroll
                for (int r = 0; r < 3; ++r) pd[r] = u32x4{0u, 0u, 0u, 0u};
                // tap s = 0 of the previous step: its dy fragment moved one pixel up; `first` = first dword
                // of this lane's packet of the step after it
                auto left_tap = [&](uint32_t first) {
                    const auto sw = __builtin_amdgcn_permlane32_swap(pav[0], first, false, false);
                    const uint32_t after = khalf ? sw[0] : sw[1];
                    const u32x4 a0 = {__builtin_amdgcn_alignbit(pav[1], pav[0], 16),
                                      __builtin_amdgcn_alignbit(pav[2], pav[1], 16),
                                      __builtin_amdgcn_alignbit(pav[3], pav[2], 16),
                                      __builtin_amdgcn_alignbit(after, pav[3], 16)};
#pragma unroll
                    for (int r = 0; r < 3; ++r)
                        acc[r * 3 + 0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, a0), __builtin_bit_cast(bf16x8, pd[r]), acc[r * 3 + 0], 0, 0, 0);
                };
                for (int st = 0; st < p.steps; ++st) {
                    const u32x4 av = *reinterpret_cast<const u32x4*>(a_base + st * 32);
                    u32x4 d[3];
#pragma unroll
                    for (int r = 0; r < 3; ++r)   // columns q0 + 8h .. + 7 of the lane's channel
                        d[r] = *reinterpret_cast<const u32x4*>(rowp[r] + st * 32);
                    if (st > 0) left_tap(av[0]);
                    // tap s = 2: dy one pixel down; the dword before the packet is the partner's last
                    // dword, of the previous step for the lower half (zero before the first: dy[-1])
                    const auto sm = __builtin_amdgcn_permlane32_swap(pav[3], av[3], false, false);
                    const uint32_t before = khalf ? sm[0] : sm[1];
                    const u32x4 a2 = {__builtin_amdgcn_alignbit(av[0], before, 16),
                                      __builtin_amdgcn_alignbit(av[1], av[0], 16),
                                      __builtin_amdgcn_alignbit(av[2], av[1], 16),
                                      __builtin_amdgcn_alignbit(av[3], av[2], 16)};
#pragma unroll
                    for (int r = 0; r < 3; ++r) {
                        acc[r * 3 + 1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, av), __builtin_bit_cast(bf16x8, d[r]), acc[r * 3 + 1], 0, 0, 0);
                        acc[r * 3 + 2] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(bf16x8, a2), __builtin_bit_cast(bf16x8, d[r]), acc[r * 3 + 2], 0, 0, 0);
                    }
                    if (do_db) dbacc += sum8(av);
                    pav = av;
#pragma unroll
                    for (int r = 0; r < 3; ++r) pd[r] = d[r];
                }
                // tap s = 0 of the last step: past its upper half lies dy pixel 16 * steps, beyond the row
                left_tap(0u);
            }
            // the next step's rows go to the ring slot nobody reads now and to the other dy buffer
            store_step(pe & 3, dbuf ^ 1);
            __syncthreads();
            dbuf ^= 1;
            pe += 1; g += 1;
            if (g >= g1) break;
            if (pe > p.P + 1) {              // image done: the next output row is row 0 of image n + 1
                n += 1; pe = -1; g -= 3;     // three steps fill the ring again before that row is multiplied
            }
        }
    }

    // ---- partial tile [split][tap][k][c]; the wavefronts of k rows / channels that do not exist write nothing
    const int CRS = p.C * 9;
    float* __restrict__ out = p.out + (size_t)worker * p.K * CRS;
    const int c = c0 + wc * 32 + (lane & 31);
    if (c < p.C) {
#pragma unroll
        for (int t = 0; t < 9; ++t)
#pragma unroll
            for (int e = 0; e < 16; ++e) {
                const int k = k0 + wk * 32 + (e >> 2) * 8 + khalf * 4 + (e & 3);
                if (k < p.K) out[((size_t)t * p.K + k) * p.C + c] = acc[t][e];
            }
    }
    if (do_db) {   // lanes l and l + 32 hold the two 8-pixel halves of row l's 16-pixel steps
        const float tot = dbacc + __shfl_xor(dbacc, 32);
        const int k = k0 + wk * 32 + (lane & 31);
        if (khalf == 0 && k < p.K) p.db_out[(size_t)worker * p.K + k] = tot;
    }
}

}  // namespace

// 3x3 / stride 1 / pad 1 bf16 layers whose rows are whole 16-byte packets and fit the LDS budget.
// On success *workers is the number of splits (partial tiles) the kernel writes.
bool wgrad_rows_bf16_applies(const ConvGeom& g, int* workers) {
    if (g.R != 3 || g.S != 3 || g.sh != 1 || g.sw != 1 || g.ph != 1 || g.pw != 1) return false;
    if ((g.W & 7) || (g.Q & 7) || (g.x_ns & 7) || (g.y_ns & 7) || g.C < 32 || g.K < 32) return false;
    const long long xb = ((long long)(g.N - 1) * g.x_ns + (long long)g.C * g.H * g.W) * 2;
    const long long dyb = ((long long)(g.N - 1) * g.y_ns + (long long)g.K * g.P * g.Q) * 2;
    if (xb >= 0x7fffffffLL || dyb >= 0x7fffffffLL) return false;
    if (CT * (g.W / 8) > LOADS * 256 || KT * (g.Q / 8) > LOADS * 256) return false;
    const int xpitch = row_pitch((ORG + g.W + 8) * 2), dypitch = row_pitch(((g.Q + 15) / 16 * 16) * 2);
    if (4 * CT * xpitch + 2 * KT * dypitch > 80 * 1024) return false;
    const int groups = ((g.K + KT - 1) / KT) * ((g.C + CT - 1) / CT);
    int w = 512 / groups / 8 * 8;            // two workgroups per CU in all, whole XCD rounds
    if (w < 8) return false;
    const long long rows = (long long)g.N * g.P;
    while (w > 8 && rows / w < 8) w -= 8;   // keep the three ring-filling steps of a range a small part of it
    *workers = w;
    return true;
}

hipError_t launch_wgrad_rows_bf16(const ConvGeom& g, int workers, const void* x, const void* dy, float* partials,
                                  float* db_partials, hipStream_t st) {
    RowsWgradParams p{};
    p.x = (const uint16_t*)x; p.dy = (const uint16_t*)dy; p.out = partials; p.db_out = db_partials;
    p.N = g.N; p.C = g.C; p.H = g.H; p.W = g.W; p.K = g.K; p.P = g.P; p.Q = g.Q;
    p.x_ns = g.x_ns; p.dy_ns = g.y_ns;
    p.x_bytes = (unsigned)(((long long)(g.N - 1) * g.x_ns + (long long)g.C * g.H * g.W) * 2);
    p.dy_bytes = (unsigned)(((long long)(g.N - 1) * g.y_ns + (long long)g.K * g.P * g.Q) * 2);
    p.k_groups = (g.K + KT - 1) / KT; p.c_groups = (g.C + CT - 1) / CT; p.workers = workers;
    p.rows_total = g.N * g.P;
    p.rows_per_worker = (p.rows_total + workers - 1) / workers;
    p.xpitch = row_pitch((ORG + g.W + 8) * 2);
    p.dypitch = row_pitch(((g.Q + 15) / 16 * 16) * 2);
    p.xchunks = g.W / 8; p.dychunks = g.Q / 8;
    p.steps = (g.Q + 15) / 16;
    p.x_rounds = (CT * p.xchunks + 255) / 256; p.d_rounds = (KT * p.dychunks + 255) / 256;
    p.div_p = make_fastdiv(g.P); p.div_xchunks = make_fastdiv(p.xchunks); p.div_dychunks = make_fastdiv(p.dychunks);
    const size_t lds = (size_t)4 * CT * p.xpitch + (size_t)2 * KT * p.dypitch;
    if (lds > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(wgrad_rows3x3_bf16_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    ProbeScope probe(st);
    (void)hipGetLastError();
    hipLaunchKernelGGL(wgrad_rows3x3_bf16_kernel, dim3((unsigned)(p.k_groups * p.c_groups * workers)), dim3(256), lds, st, p);
    return hipGetLastError();
}

}  // namespace purine

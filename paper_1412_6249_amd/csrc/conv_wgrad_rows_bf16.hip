// bf16 weight gradient for 3x3 / stride 1 / pad 1 layers with rows of whole 16-byte packets
// (ConvBwdWeight of paper Figure 1(b)):
//
//     dw[k, c, r, s] = sum over (n, p, q) of dy[n, k, p, q] * x[n, c, p - 1 + r, q - 1 + s]
//
// The reduction runs over pixels, and NCHW keeps the pixels of a row contiguous, so BOTH MFMA
// operands (8 consecutive reduction elements per lane) are 16-byte windows of rows as they lie in
// memory. A workgroup walks over output rows; per row it holds in LDS, in their natural layout, the
// dy row of its 64 output channels and a ring of the input rows of its 64 input channels
// (consecutive output rows share two of their three input rows, so each step brings in ONE new
// input row and one dy row). The rows come in by loads that write LDS directly, requested two
// steps ahead. The three column taps are had by shifting the dy fragment one pixel either way in
// registers (funnel shifts; the neighbouring dword comes from the partner lane's registers), the
// input rows' packets serve all taps as they are: a step of 16 pixels costs a wavefront 4 LDS reads
// for 9 MFMAs. Each wavefront owns 32 output channels x 32 input channels x all nine taps (144
// accumulators). Workgroups are persistent over a contiguous range of (image, row) pairs; their
// fp32 partial tiles go to scratch as [split][tap][k][c] and the fixed-order second pass of the
// general kernel adds them.
#include "common.h"
#include <type_traits>

namespace purine {
namespace {

typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int KT = 64, CT = 64;     // output / input channels per workgroup
constexpr int ORG = 8;              // element of an x row in LDS that holds image column 0
constexpr int PITCH = 144;          // LDS bytes per staged row: 9 packets of 16 bytes (see row_pitch)
constexpr int SLOT = 64 * PITCH;    // one staged row of each of 64 channels: 576 packets = 9 wavefront loads
constexpr int XSLOTS = 5, DSLOTS = 3;   // rows being read (3 / 1) + rows in flight (2 / 2)
constexpr int RQ = 5;               // loads per wavefront and step: two wavefronts share a slot's 9
constexpr int LDS_BYTES = (XSLOTS + DSLOTS) * SLOT + 1024;   // + 1 KB that takes the loads nobody needs

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
    int xchunks, dychunks;             // 16-byte packets per x row (W / 8) and dy row (Q / 8)
    int steps;                         // 16-pixel MFMA steps per output row: ceil(Q / 16)
    FastDiv div_p;
};

__device__ __forceinline__ float sum8(const u32x4 u) {
    float s = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) s += __uint_as_float(u[i] << 16) + __uint_as_float(u[i] & 0xffff0000u);
    return s;
}

__global__ __launch_bounds__(256, 2) void wgrad_rows3x3_bf16_kernel(const RowsWgradParams p) {
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    unsigned char* xs = smem;                                   // [XSLOTS][CT] rows of PITCH bytes
    unsigned char* dys = smem + XSLOTS * SLOT;                  // [DSLOTS][KT] rows of PITCH bytes
    unsigned char* spare = smem + (XSLOTS + DSLOTS) * SLOT;     // 1 KB

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
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

    // ---- once: zero everything
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < LDS_BYTES / 16; i += 256) *reinterpret_cast<u32x4*>(smem + i * 16) = z;
    }

    // ---- Rows come in by loads that write LDS directly (no registers, so requests can run two steps
    // ahead beside 144 accumulators). One such load of a wavefront fills 64 consecutive 16-byte
    // packets of LDS, lane l the l-th, with the 16 bytes at the lane's own buffer offset, or with
    // zeros when that offset lies outside the buffer. A staged row is 9 packets (x: a halo packet,
    // up to 7 of data, zeros; dy: up to 7 of data, zeros), a slot 576 packets = 9 loads: wavefronts 0
    // and 1 share the x slot's loads (t = parity, parity + 2, ...), wavefronts 2 and 3 the dy slot's.
    // The lanes of halo / tail packets and of channels that do not exist keep an offset outside the
    // buffer, which is also how rows above and below the image become zeros. A wavefront issues RQ
    // loads per step whatever happens (those nobody needs go to the spare KB), so that a wait can
    // count them.
    const bool loads_x = wave < 2;
    const int parity = wave & 1;
    int goff[RQ];
#pragma unroll
    for (int i = 0; i < RQ; ++i) {
        const int t = parity + 2 * i;
        const int pk = t * 64 + lane;
        const int row = pk / 9, jp = pk - row * 9;
        if (loads_x) {
            const bool ok = t < 9 && c0 + row < p.C && jp >= 1 && jp <= p.xchunks;     // packet 0: the ORG elements
            goff[i] = ok ? ((c0 + row) * p.H * p.W + (jp - 1) * 8) * 2 : -1;
        } else {
            const bool ok = t < 9 && k0 + row < p.K && jp < p.dychunks;
            goff[i] = ok ? ((k0 + row) * p.P * p.Q + jp * 8) * 2 : -1;
        }
    }
    // (the descriptor has to sit in scalar registers: say so, or every load becomes a loop over lanes)
    const uint64_t src = reinterpret_cast<uint64_t>(loads_x ? p.x : p.dy);
    // (readfirstlane returns a signed int: through uint32_t, or the low word's top bit smears over the high word)
    const uint32_t src_lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)src);
    const uint32_t src_hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(src >> 32));
    const uint64_t src_u = ((uint64_t)src_hi << 32) | (uint64_t)src_lo;
    const __amdgpu_buffer_rsrc_t rs = __builtin_amdgcn_make_buffer_rsrc(
        reinterpret_cast<uint16_t*>(src_u), (short)0,
        __builtin_amdgcn_readfirstlane((int)(loads_x ? p.x_bytes : p.dy_bytes)), 0x00020000);
    // this wavefront's share of: input row h of image n into x slot `xslot`, dy row pp into dy slot `dslot`
    // (zeros when the row is outside the image / when !real_dy); !exists: nothing needed
    auto request = [&](bool exists, int n, int h, bool real_dy, int pp, int xslot, int dslot) {
        const bool row_ok = exists && (loads_x ? (unsigned)h < (unsigned)p.H : real_dy);
        const int base = loads_x ? n * p.x_ns * 2 + h * p.W * 2 : n * p.dy_ns * 2 + pp * p.Q * 2;
        unsigned char* slot = loads_x ? xs + xslot * SLOT : dys + dslot * SLOT;
#pragma unroll
        for (int i = 0; i < RQ; ++i) {
            const int t = parity + 2 * i;
            const unsigned v = (row_ok && goff[i] >= 0) ? (unsigned)(base + goff[i]) : 0x80000000u;
            unsigned char* dst = (exists && t < 9) ? slot + t * 1024 : spare;
            __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (__attribute__((address_space(3))) void*)dst, 16, v, 0, 0, 0);
        }
    };
    // every load of this wavefront but the `newest` youngest has written its packets; then all
    // wavefronts meet. No fence: one would wait for the loads in flight as well. The empty asm
    // statements keep the compiler from moving LDS accesses across.
    auto rows_landed = [&](auto newest) {
        asm volatile("" ::: "memory");
        __builtin_amdgcn_s_waitcnt(0x0070 | decltype(newest)::value);      // vmcnt(newest), lgkmcnt(0)
        __builtin_amdgcn_s_barrier();
        asm volatile("" ::: "memory");
    };

    floatx16 acc[9];
#pragma unroll
    for (int t = 0; t < 9; ++t)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc[t][e] = 0.0f;
    float dbacc = 0.0f;
    const bool do_db = p.db_out != nullptr && c0 == 0 && wc == 0;

    if (g0 < g1) {
        // Extended row index pe of an image runs from -1 to P + 1: step pe brings in input row pe and
        // the dy row of step pe + 1, and multiplies output row pe - 2 (when that row exists and
        // belongs to this worker) with input rows pe - 3 .. pe - 1. The first three steps of a range
        // only fill the ring. Step k's rows are requested at the start of step k - 1 and must have
        // landed at the end of step k: two steps' requests are in flight.
        struct Pos { int n, pe, g; };        // image, extended row, flattened output row the step multiplies
        auto advance = [&](Pos& s) -> bool {
            s.pe += 1; s.g += 1;
            if (s.g >= g1) return false;
            if (s.pe > p.P + 1) {            // image done: the next output row is row 0 of image n + 1
                s.n += 1; s.pe = -1; s.g -= 3;   // three steps fill the ring again before that row is multiplied
            }
            return true;
        };
        // the rows step s brings in: input row pe, dy row of output row (pe + 1) - 2 = pe - 1
        auto request_for = [&](const Pos& s, bool exists, int xslot, int dslot) {
            const bool dy_real = s.pe - 1 >= 0 && s.pe - 1 < p.P && s.g + 1 >= g0 && s.g + 1 < g1;
            request(exists, s.n, s.pe, dy_real, s.pe - 1, xslot, dslot);
        };
        Pos cur;
        cur.n = fastdiv(g0, p.div_p);
        cur.pe = g0 - cur.n * p.P - 1;       // first step: brings in row p0 - 1, multiplies nothing
        cur.g = g0 - 3;
        Pos nxt = cur;
        bool has_next = advance(nxt);
        int kx = 0, kd = 0;                  // step number mod XSLOTS / mod DSLOTS: the slots of this step's rows
        __syncthreads();                     // zeros in place
        request_for(cur, true, 0, 0);
        while (true) {
            const int kx1 = kx + 1 == XSLOTS ? 0 : kx + 1, kd1 = kd + 1 == DSLOTS ? 0 : kd + 1;
            request_for(nxt, has_next, kx1, kd1);
            const int pe = cur.pe;
            const bool real = pe - 2 >= 0 && pe - 2 < p.P && cur.g >= g0;
            if (real) {
                // dy row of the step before this one; input rows of the three steps before it
                const int dprev = kd == 0 ? DSLOTS - 1 : kd - 1;
                const unsigned char* a_base = dys + dprev * SLOT + (wk * 32 + (lane & 31)) * PITCH + khalf * 16;
                const int xrow = (wc * 32 + (lane & 31)) * PITCH + (ORG + khalf * 8) * 2;   // column 8h of the lane's channel
                const unsigned char* rowp[3];
#pragma unroll
                for (int r = 0; r < 3; ++r) {
                    const int sl = kx + 2 + r;           // (k - 3 + r) mod XSLOTS
                    rowp[r] = xs + (sl >= XSLOTS ? sl - XSLOTS : sl) * SLOT + xrow;
                }
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
            // this step's rows are in LDS (the next step's, requested above, may still be in flight)
            rows_landed(std::integral_constant<int, RQ>());
            if (!has_next) break;
            cur = nxt;
            has_next = advance(nxt);
            kx = kx1; kd = kd1;
        }
        // the last step's requests (to the spare KB) must not outlive the workgroup's LDS
        __builtin_amdgcn_s_waitcnt(0x0070);
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
    // staged rows of exactly PITCH bytes: rows of at most 56 pixels
    if (row_pitch((ORG + g.W + 8) * 2) != PITCH || row_pitch(((g.Q + 15) / 16 * 16) * 2) != PITCH) return false;
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
    p.xchunks = g.W / 8; p.dychunks = g.Q / 8;
    p.steps = (g.Q + 15) / 16;
    p.div_p = make_fastdiv(g.P);
    const size_t lds = LDS_BYTES;
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

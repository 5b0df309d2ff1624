// bf16 MFMA implicit GEMM with the input patch staged in LDS (Conv / ConvBwdData of paper
// Figure 1(b), unit-stride gathers: forward with stride 1, backward-data with any stride after
// phase folding).
//
// A workgroup owns BM output rows (channels) and BN consecutive output pixels of ONE image. Those
// pixels span a few image rows; the input positions all their taps touch form a haloed patch of
// (rows spanned + Rt - 1) x (Wo + St - 1) positions. Per group of 16 gathered channels (one MFMA
// reduction step) the patch is brought into LDS ONCE, straight from the NCHW tensor: a lane loads
// 8 consecutive pixels of one channel as one 16-byte packet (coalesced along W), eight channels'
// packets are transposed in registers (one byte-permute per output dword) into eight
// [pixel][8 channels] packets and stored pixel-major, which is the operand layout the bf16 MFMA
// wants (8 consecutive reduction elements per lane). Every tap then reads its B fragments from the
// same patch at a shifted position, so the global gathers of the tap-major kernel shrink by the
// number of taps and no re-laid-out copy of the tensor ever goes to HBM. Rows and columns outside
// the image are zeros in the patch (the halo columns are cleared once, out-of-image rows come back
// as zeros from range-checked buffer loads).
//
// LDS layout of the patch. A lane of the MFMA loop owns adjacent output pixels (so that its stores
// are whole packets), hence the lanes of one fragment read are TWO patch positions apart. The patch
// therefore keeps four planes, (position parity, 8-channel half), each holding the 16-byte packets
// of positions P with index P >> 1: a fragment read covers consecutive packets of one plane and
// has no bank conflict whatever the tap's shift. Plane sizes are 32 bytes past a multiple of 128,
// which keeps the fill's stores (four consecutive 8-pixel packets x two halves per 8 lanes) down to
// a two-way conflict. The filter rows use the same idea: [tap][half][row] packets.
//
// The filter of the same 16 channels sits beside the patch for ALL taps of a stage (from a copy
// repacked to A[group][tap][i][16]), so the tap loop runs without barriers: one stage = one channel
// group x a run of taps, two barriers per stage. The loads of the next stage (filter and, when
// the group changes, patch) are issued before the stage's MFMAs and land in registers meanwhile.
// Accumulators stay in registers for the whole reduction.
#include "pix_common.h"

namespace purine {
namespace pix {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef unsigned u32x4 __attribute__((ext_vector_type(4)));

constexpr int GC = 16;              // gathered channels per group: one MFMA reduction step
constexpr int A_ROUNDS = 8;         // 16-byte filter pieces per thread and stage, at most

// ROUNDS: patch fill tasks (8 channels x 8 pixels each) per thread and channel group.
template <bool MINUS, bool D2S, bool FUSED, int TM, int TN, int WM, int WN, int ROUNDS>
__global__ __launch_bounds__(256, 2) void igemm_patch_bf16_kernel(const PixParams p, const PatchGeom q) {
    constexpr int NT = WM * WN * 64;
    constexpr int BM = WM * TM * 32;
    constexpr int BN = WN * TN * 32;
    static_assert(NT == 256, "four wavefronts");

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* bias_s = reinterpret_cast<float*>(smem);                 // [BM]
    unsigned char* As = smem + BM * 4;                              // [taps per stage][half][BM] 16-byte packets
    unsigned char* patch = As + q.a_bytes;                          // [parity][half][position >> 1] 16-byte packets
    const int PB = q.plane_bytes;
    const int APB = BM * 16 + 64;                                   // filter plane (one half of one tap)
    // byte offset of position P, half h
    auto patch_at = [&](int P, int h) { return ((P & 1) * 2 + h) * PB + (P >> 1) * 16; };

    const uint16_t* __restrict__ in = (const uint16_t*)p.in;
    const uint16_t* __restrict__ wt = (const uint16_t*)p.wt;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave / WN, wn = wave % WN;

    const int tile = xcd_tile(blockIdx.x, p.tiles_i * p.tiles_pix);
    const int i0 = (tile % p.tiles_i) * BM;
    const int tp = tile / p.tiles_i;
    const int n = fastdiv(tp, q.div_tpi);
    const int pix0 = (tp - n * q.tiles_per_img) * BN;          // first pixel of the tile inside image n
    const int pix_end = min(pix0 + BN, p.HoWo);
    const int ho_first = fastdiv(pix0, p.div_wo);
    const int h_lo = ho_first + q.h_lo_add;

    // ---- patch fill tasks of this thread: (patch row, 8-channel half of the group, 8-pixel packet)
    // Task t: 4 consecutive packets (t & 3), half (t >> 2) & 1, then the row's remaining packet quads, then rows.
    unsigned g_voff[ROUNDS];   // byte offset of the packet in the half's first channel of group 0 (2^31: row outside the image)
    int l_even[ROUNDS];        // patch byte offsets of the packet's pixels 0 and 1 (pixels 2j, 2j + 1 follow at
    int l_odd[ROUNDS];         // 16 * j); a thread without a task in this round writes into the spare packets
    int l_step[ROUNDS];        // behind the planes (step 0): no branch around the stores
    int cg8[ROUNDS];
#pragma unroll
    for (int r = 0; r < ROUNDS; ++r) {
        const int t = tid + r * NT;
        const int pr = fastdiv(t, q.div_tpr);
        const int u = t - pr * q.tasks_per_row;
        const int cg = (u >> 2) & 1;
        const int chunk = (u >> 3) * 4 + (u & 3);
        const bool live = pr < q.pr_max && chunk < q.chunks;
        const int hi = h_lo + pr;
        const bool row_ok = live & ((unsigned)hi < (unsigned)p.Hi);
        g_voff[r] = row_ok ? (unsigned)(n * p.in_ns + cg * 8 * p.HiWi + hi * p.Wi + chunk * 8) * 2u : 0x80000000u;
        const int P0 = pr * q.pw + chunk * 8 - q.w_lo;
        l_even[r] = live ? patch_at(P0, cg) : 4 * PB + (tid & 7) * 16;
        l_odd[r] = live ? patch_at(P0 + 1, cg) : 4 * PB + (tid & 7) * 16;
        l_step[r] = live ? 16 : 0;
        cg8[r] = cg * 8;
    }
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(in), (short)0, (int)p.in_bytes, 0x00020000);

    u32x4 pre[ROUNDS][8];      // the packets of the next channel group, as loaded (channel-major)
    auto load_patch = [&](int c0) {
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const unsigned v = (c0 + cg8[r] < p.Ci) ? g_voff[r] : 0x80000000u;   // padding channels read as zeros
#pragma unroll
            for (int e = 0; e < 8; ++e)
                pre[r][e] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, v, (c0 + e) * p.HiWi * 2, 0);
        }
    };
    auto store_patch = [&]() {
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
#pragma unroll
            for (int px = 0; px < 8; ++px) {
                // pixel px of the packet: channel pairs (0,1) (2,3) (4,5) (6,7), low or high halves of dword px/2
                const unsigned sel = (px & 1) ? 0x07060302u : 0x05040100u;
                u32x4 o;
#pragma unroll
                for (int c2 = 0; c2 < 4; ++c2)
                    o[c2] = __builtin_amdgcn_perm(pre[r][2 * c2 + 1][px >> 1], pre[r][2 * c2][px >> 1], sel);
                *reinterpret_cast<u32x4*>(patch + ((px & 1) ? l_odd[r] : l_even[r]) + (px >> 1) * l_step[r]) = o;
            }
        }
    };

    // ---- filter pieces served by this thread: piece f of a stage = (tap of the stage, row, 8-channel half).
    // Source offsets are relative to the stage's first tap in A[group][tap][i_pad][16].
    const int n_taps = p.Rt * p.St;
    const int n_groups = p.Ci_pad / GC;
    const int tc = q.taps_per_stage;
    const int n_chunks = (n_taps + tc - 1) / tc;
    const int n_stages = n_groups * n_chunks;
    int a_src[A_ROUNDS], a_dst[A_ROUNDS];
#pragma unroll
    for (int it = 0; it < A_ROUNDS; ++it) {
        const int f = tid + it * NT;
        const int tap = f / (BM * 2), rem = f - tap * (BM * 2);
        const int row = rem >> 1, half = rem & 1;
        const bool live = tap < tc;
        a_src[it] = live ? (tap * p.i_pad + i0 + row) * GC + half * 8 : -1;
        a_dst[it] = live ? (tap * 2 + half) * APB + row * 16 : BM * 16 + (tid & 3) * 16;   // parked in a plane's spare bytes
    }
    u32x4 a_reg[A_ROUNDS];
    auto load_a = [&](int group, int t0, int nt) {
        const int base = (group * n_taps + t0) * p.i_pad * GC;
        const int limit = nt * p.i_pad * GC;                    // taps past the stage's last one re-read piece 0
#pragma unroll
        for (int it = 0; it < A_ROUNDS; ++it) {
            if (it >= q.a_rounds) break;                        // uniform: rounds this tile shape never needs
            const int off = (a_src[it] >= 0 && a_src[it] < limit) ? a_src[it] : 0;
            a_reg[it] = *reinterpret_cast<const u32x4*>(wt + base + off);
        }
    };
    auto store_a = [&]() {
#pragma unroll
        for (int it = 0; it < A_ROUNDS; ++it) {
            if (it >= q.a_rounds) break;
            *reinterpret_cast<u32x4*>(As + a_dst[it]) = a_reg[it];
        }
    };

    // ---- this lane's B-fragment positions (byte offsets into the patch at tap (0,0)); columns past the
    // tile's last pixel re-read that pixel (their results are never stored)
    // position P = P_lane + shift sits at half * PB + 8 * P + (P & 1) * (2 * PB - 8): one base per parity of the shift
    int b_same[TN], b_flip[TN];
#pragma unroll
    for (int b = 0; b < TN; ++b) {
        const int pix = min(pix0 + wn * TN * 32 + TN * (lane & 31) + b, pix_end - 1);   // a lane's tiles: adjacent pixels
        const int ho = fastdiv(pix, p.div_wo);
        const int wo = pix - ho * p.Wo;
        const int P = (ho - ho_first) * q.pw + wo + q.pos_add;
        const int lin = (lane >> 5) * PB + P * 8;
        b_same[b] = lin + (P & 1) * (2 * PB - 8);
        b_flip[b] = lin + ((P & 1) ^ 1) * (2 * PB - 8);
    }
    const int a_row = (lane >> 5) * APB + (wm * TM * 32 + (lane & 31)) * 16;

    floatx16 acc[TM][TN];
#pragma unroll
    for (int a = 0; a < TM; ++a)
#pragma unroll
        for (int b = 0; b < TN; ++b)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;

    // ---- prologue: first stage's loads, halo columns to zero
    load_patch(0);
    load_a(0, 0, min(tc, n_taps));
    {
        const int halo_w = q.halo_l + q.pw - q.halo_r0;        // halo columns per patch row
        const int total = q.pr_max * halo_w * (GC / 8);
        for (int i = tid; i < total; i += NT) {
            const int half = i & 1;
            const int hp = i >> 1;
            const int pr = fastdiv(hp, q.div_halo);
            const int hc = hp - pr * halo_w;
            const int pc = hc < q.halo_l ? hc : q.halo_r0 + (hc - q.halo_l);
            const u32x4 z = {0u, 0u, 0u, 0u};
            *reinterpret_cast<u32x4*>(patch + patch_at(pr * q.pw + pc, half)) = z;
        }
    }
    if (FUSED) stage_bias<uint16_t, BM, NT>(bias_s, p, i0, tid);

    int group = 0, chunk = 0;
    for (int stage = 0; stage < n_stages; ++stage) {
        // the barrier that ended the previous stage: nobody reads the filter rows or the patch any more
        if (chunk == 0) store_patch();
        store_a();
        __syncthreads();
        const int t0 = chunk * tc;
        const int nt = min(tc, n_taps - t0);
        // next stage's loads fly during this stage's MFMAs
        int nx_group = group, nx_chunk = chunk + 1;
        if (nx_chunk >= n_chunks) { nx_chunk = 0; nx_group += 1; }
        if (stage + 1 < n_stages) {
            if (nx_chunk == 0) load_patch(nx_group * GC);
            load_a(nx_group, nx_chunk * tc, min(tc, n_taps - nx_chunk * tc));
        }
        int tap_r = fastdiv(t0, q.div_st);
        int tap_s = t0 - tap_r * p.St;
        const unsigned char* asrc = As + a_row;
        for (int tap = 0; tap < nt; ++tap) {
            const int shift = tap_r * q.pw + tap_s;                 // in patch positions
            const unsigned char* bsrc = patch + (MINUS ? -shift : shift) * 8;
            const bool odd = shift & 1;
            bf16x8 av[TM], bv[TN];
#pragma unroll
            for (int a = 0; a < TM; ++a) av[a] = *reinterpret_cast<const bf16x8*>(asrc + a * 32 * 16);
#pragma unroll
            for (int b = 0; b < TN; ++b) bv[b] = *reinterpret_cast<const bf16x8*>(bsrc + (odd ? b_flip[b] : b_same[b]));
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
                    acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(av[a], bv[b], acc[a][b], 0, 0, 0);
            asrc += 2 * APB;
            tap_s += 1;
            const bool wrap = tap_s >= p.St;
            tap_s = wrap ? 0 : tap_s;
            tap_r += wrap ? 1 : 0;
        }
        __syncthreads();
        group = nx_group;
        chunk = nx_chunk;
    }

    if (!D2S && q.pairs) {
        store_adjacent<FUSED, TM, TN, !MINUS>(p, acc, i0 + wm * TM * 32, n, pix0 + wn * TN * 32 + TN * (lane & 31), pix_end,
                                              lane, bias_s, i0);
        return;
    }
    if (D2S && p.sh == 2 && p.sw == 2 && q.d2s_buffers) {
        int hq_of[TN], wq_of[TN];
        bool live_of[TN];
#pragma unroll
        for (int b = 0; b < TN; ++b) {
            const int pix = pix0 + wn * TN * 32 + TN * (lane & 31) + b;
            live_of[b] = pix < pix_end;
            hq_of[b] = fastdiv(live_of[b] ? pix : 0, p.div_wo);
            wq_of[b] = (live_of[b] ? pix : 0) - hq_of[b] * p.Wo;
        }
        store_d2s2_adjacent<FUSED, TM, TN>(p, acc, i0 + wm * TM * 32, n, hq_of, wq_of, live_of, lane);
        return;
    }
    store_tile<uint16_t, D2S, FUSED, TM, TN, !MINUS>(p, (uint16_t*)p.out, acc, i0 + wm * TM * 32,
                                                     n * p.HoWo + pix0 + wn * TN * 32 + TN * (lane & 31), lane >> 5,
                                                     bias_s, i0, n * p.HoWo + pix_end, 1);
}

// ---- the same computation with the wavefronts of a workgroup split into two roles ----------------
// Eight wavefronts, one workgroup per CU, persistent over pixel tiles of BM rows x 512 pixels.
// Wavefronts 4-7 ("fill") bring the next stages' patch and filter rows from global memory into
// registers, transpose, and store them into the OTHER of two LDS buffers; wavefronts 0-3
// ("multiply") run the current stage (one 16-channel group, all taps) and, after a tile's last
// stage, its epilogue. One barrier per stage hands a buffer over in each direction.
//
// A multiply lane owns FOUR adjacent pixels, and the patch is kept as eight planes (position mod 4,
// 8-channel half) of 16-byte packets. The B fragments of a filter row's taps are then a sliding
// window: pixel b at column tap s reads position base + b + s, so a row of ST taps needs 4 + ST - 1
// fragment reads instead of 4 * ST, and with the filter rows read once per tap for all four pixel
// tiles the LDS traffic per MFMA is half that of the one-role kernel, whose tap loop is bound by it.
// Rows are taken in pairs, the next row's fragments requested before the current row's MFMAs.
// Pixel tiles count in rows of q.wv pixels, the output width rounded up to a multiple of four, so
// that a lane's four pixels share an output row; the up to three pixels past a row's end are
// computed and not stored (only the depth-to-space epilogue of stride-2 layers takes such widths).
constexpr int RTN = 4;     // adjacent pixels per multiply lane
template <bool MINUS, bool D2S, bool FUSED, int TM, int ST, int ROUNDS>
__global__ __launch_bounds__(512, 1) void igemm_patch_roles_bf16_kernel(const PixParams p, const PatchGeom q) {
    constexpr int NT = 256;                 // threads of each role
    constexpr int TN = RTN;
    constexpr int BM = TM * 32;
    constexpr int BN = 4 * TN * 32;         // four multiply wavefronts side by side
    constexpr int NWIN = TN + ST - 1;

    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float* bias_s = reinterpret_cast<float*>(smem);                 // [i_pad]: every row tile's bias
    const int PB = q.plane_bytes;
    const int patch_bytes = 2 * TN * PB + 128;
    const int buf_bytes = q.a_bytes + patch_bytes;                  // one stage: filter rows, then the patch
    unsigned char* buf0 = smem + p.i_pad * 4;
    const int APB = BM * 16 + 64;
    // byte offset of position P, half h
    auto patch_at = [&](int P, int h) { return ((P & (TN - 1)) * 2 + h) * PB + (P >> 2) * 16; };

    const uint16_t* __restrict__ in = (const uint16_t*)p.in;
    const uint16_t* __restrict__ wt = (const uint16_t*)p.wt;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int rt = tid & (NT - 1);          // thread index inside its role

    // once: both buffers to zero (halo columns are never written again: fill tasks write image columns
    // only, and rows outside the image arrive as zeros), every row tile's bias
    {
        const u32x4 z = {0u, 0u, 0u, 0u};
        for (int i = tid; i < 2 * buf_bytes / 16; i += 512) *reinterpret_cast<u32x4*>(buf0 + i * 16) = z;
        if (FUSED) {
            const uint16_t* __restrict__ bias = (const uint16_t*)p.bias;
            if (bias)
                for (int r = tid; r < p.i_pad; r += 512) bias_s[r] = r < p.Co ? Elem<uint16_t>::load(bias, r) : 0.0f;
        }
    }
    __syncthreads();

    // this workgroup's tiles: logical index w (contiguous inside an XCD), tiles w, w + G, w + 2G, ...
    const int G = gridDim.x;
    const int total = p.tiles_i * p.tiles_pix;
    const int w_id = (G & 7) == 0 ? ((int)blockIdx.x & 7) * (G >> 3) + ((int)blockIdx.x >> 3) : (int)blockIdx.x;
    const int my_tiles = w_id < total ? (total - 1 - w_id) / G + 1 : 0;
    const int n_taps = p.Rt * ST;
    const int n_groups = p.Ci_pad / GC;
    const int n_stages = my_tiles * n_groups;

    if (wave >= 4) {
        // ================= fill role =================
        unsigned g_voff[ROUNDS];
        int l_off[ROUNDS][4], l_step[ROUNDS], cg8[ROUNDS], t_pr[ROUNDS], t_chunk[ROUNDS];
        bool t_live[ROUNDS];
#pragma unroll
        for (int r = 0; r < ROUNDS; ++r) {
            const int t = rt + r * NT;
            const int pr = fastdiv(t, q.div_tpr);
            const int u = t - pr * q.tasks_per_row;
            const int cg = (u >> 2) & 1;
            const int chunk = (u >> 3) * 4 + (u & 3);
            const bool live = pr < q.pr_max && chunk < q.chunks;
            const int P0 = pr * q.pw + chunk * 8 - q.w_lo;
            // pixels px and px + 4 of the packet share a plane, 16 bytes apart; a thread without a task
            // writes into the spare packets behind the planes
#pragma unroll
            for (int px = 0; px < 4; ++px) l_off[r][px] = live ? patch_at(P0 + px, cg) : 2 * TN * PB + (rt & 7) * 16;
            l_step[r] = live ? 16 : 0;
            cg8[r] = cg * 8;
            t_pr[r] = pr; t_chunk[r] = chunk; t_live[r] = live;
            g_voff[r] = 0x80000000u;
        }
        const __amdgpu_buffer_rsrc_t rsrc =
            __builtin_amdgcn_make_buffer_rsrc(const_cast<uint16_t*>(in), (short)0, (int)p.in_bytes, 0x00020000);
        int a_src[A_ROUNDS], a_dst[A_ROUNDS];
#pragma unroll
        for (int it = 0; it < A_ROUNDS; ++it) {
            const int f = rt + it * NT;
            const int tap = f / (BM * 2), rem = f - tap * (BM * 2);
            const int row = rem >> 1, half = rem & 1;
            const bool live = tap < n_taps;
            a_src[it] = live ? (tap * p.i_pad + row) * GC + half * 8 : -1;      // + i0 * GC per tile
            a_dst[it] = live ? (tap * 2 + half) * APB + row * 16 : BM * 16 + (rt & 3) * 16;
        }
        // DEPTH stages of requests are in flight at any time (one register set each)
        constexpr int DEPTH = 2;
        u32x4 pre[DEPTH][ROUNDS][8];
        u32x4 a_reg[DEPTH][A_ROUNDS];
        int i0 = 0;
        int rq_group = 0, rq_tl = 0;
        // requests of the next stage in order into one register set; `real` (uniform) = false past the
        // workgroup's last stage: the same instructions, out of range (no memory traffic) or at offset 0
        auto request = [&](u32x4 (&pr)[ROUNDS][8], u32x4 (&ar)[A_ROUNDS], bool real) {
            if (rq_group == 0) {
                const int tile = min(w_id + rq_tl * G, total - 1);   // (stages past the last: any valid tile)
                i0 = (tile % p.tiles_i) * BM;
                const int tp = tile / p.tiles_i;
                const int n = fastdiv(tp, q.div_tpi);
                const int pix0 = (tp - n * q.tiles_per_img) * BN;
                const int h_lo = fastdiv(pix0, q.div_wv) + q.h_lo_add;
#pragma unroll
                for (int r = 0; r < ROUNDS; ++r) {
                    const int hi = h_lo + t_pr[r];
                    const bool row_ok = t_live[r] & ((unsigned)hi < (unsigned)p.Hi);
                    g_voff[r] = row_ok ? (unsigned)(n * p.in_ns + cg8[r] * p.HiWi + hi * p.Wi + t_chunk[r] * 8) * 2u : 0x80000000u;
                }
            }
            const int group = rq_group;
            const int c0 = group * GC;
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r) {
                const unsigned v = (real && c0 + cg8[r] < p.Ci) ? g_voff[r] : 0x80000000u;   // padding channels read as zeros
#pragma unroll
                for (int e = 0; e < 8; ++e)
                    pr[r][e] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, v, (c0 + e) * p.HiWi * 2, 0);
            }
            const int base = real ? (group * n_taps * p.i_pad + i0) * GC : 0;
#pragma unroll
            for (int it = 0; it < A_ROUNDS; ++it) {
                if (it >= q.a_rounds) break;                        // uniform
                const int off = (real && a_src[it] >= 0) ? a_src[it] : 0;
                ar[it] = *reinterpret_cast<const u32x4*>(wt + base + off);
            }
            rq_group += 1;
            if (rq_group == n_groups) { rq_group = 0; rq_tl += 1; }
        };
        auto deposit = [&](unsigned char* buf, const u32x4 (&pr)[ROUNDS][8], const u32x4 (&ar)[A_ROUNDS]) {
            unsigned char* patch = buf + q.a_bytes;
#pragma unroll
            for (int r = 0; r < ROUNDS; ++r) {
#pragma unroll
                for (int px = 0; px < 8; ++px) {
                    // pixel px of the packet: channel pairs (0,1) (2,3) (4,5) (6,7), low or high halves of dword px/2
                    const unsigned sel = (px & 1) ? 0x07060302u : 0x05040100u;
                    u32x4 o;
#pragma unroll
                    for (int c2 = 0; c2 < 4; ++c2)
                        o[c2] = __builtin_amdgcn_perm(pr[r][2 * c2 + 1][px >> 1], pr[r][2 * c2][px >> 1], sel);
                    *reinterpret_cast<u32x4*>(patch + l_off[r][px & 3] + (px >> 2) * l_step[r]) = o;
                }
            }
#pragma unroll
            for (int it = 0; it < A_ROUNDS; ++it) {
                if (it >= q.a_rounds) break;
                *reinterpret_cast<u32x4*>(buf + a_dst[it]) = ar[it];
            }
        };
        // stages 0 .. DEPTH-1 requested up front; then, per stage: deposit its set, request stage
        // s + DEPTH into the same set, barrier. Whole rounds of DEPTH stages first (every trip issues the
        // same instructions, so the waits stay counted), then the remaining stages one by one.
#pragma unroll
        for (int j = 0; j < DEPTH; ++j) request(pre[j], a_reg[j], j < n_stages);
        int s = 0;
        for (; s + DEPTH <= n_stages; s += DEPTH) {
#pragma unroll
            for (int j = 0; j < DEPTH; ++j) {
                deposit(buf0 + ((s + j) & 1) * buf_bytes, pre[j], a_reg[j]);
                request(pre[j], a_reg[j], s + j + DEPTH < n_stages);
                __syncthreads();             // stage s + j is in place; the multiply role is done with the other buffer
            }
        }
#pragma unroll
        for (int j = 0; j < DEPTH - 1; ++j) {
            if (s + j < n_stages) {
                deposit(buf0 + ((s + j) & 1) * buf_bytes, pre[j], a_reg[j]);
                __syncthreads();
            }
        }
        return;
    }

    // ================= multiply role =================
    const int wn = wave;
    const int a_row = (lane >> 5) * APB + (lane & 31) * 16;
    const int hPB = (lane >> 5) * PB;
    floatx16 acc[TM][TN];
    int X0 = 0;                              // patch position of this lane's first pixel at tap (0, 0)
    int woff[NWIN];                          // byte offsets of the window's elements in filter row 0 (plane, half, quad)
    int i0 = 0, n = 0, pix0 = 0, pix_end = 0;
    int group = 0, tl = 0;
    struct RowFrags { bf16x8 a[ST][TM]; bf16x8 w[NWIN]; };
    for (int s = 0; s < n_stages; ++s) {
        if (group == 0) {
            const int tile = w_id + tl * G;
            i0 = (tile % p.tiles_i) * BM;
            const int tp = tile / p.tiles_i;
            n = fastdiv(tp, q.div_tpi);
            pix0 = (tp - n * q.tiles_per_img) * BN;
            pix_end = min(pix0 + BN, p.Ho * q.wv);
            const int ho_first = fastdiv(pix0, q.div_wv);
            // lanes past the tile's last pixel re-read its last four (their results are never stored)
            const int pix = min(pix0 + wn * TN * 32 + TN * (lane & 31), pix_end - TN);
            const int ho = fastdiv(pix, q.div_wv);
            const int wo = pix - ho * q.wv;
            X0 = (ho - ho_first) * q.pw + wo + q.pos_add;
#pragma unroll
            for (int j = 0; j < NWIN; ++j) {
                const int X = X0 + j - (MINUS ? ST - 1 : 0);
                woff[j] = hPB + (X & (TN - 1)) * 2 * PB + (X >> 2) * 16;
            }
#pragma unroll
            for (int a = 0; a < TM; ++a)
#pragma unroll
                for (int b = 0; b < TN; ++b)
#pragma unroll
                    for (int e = 0; e < 16; ++e) acc[a][b][e] = 0.0f;
        }
        __syncthreads();                     // stage s is in place
        const unsigned char* As = buf0 + (s & 1) * buf_bytes;
        const unsigned char* patch = As + q.a_bytes;
        // `real` = false (uniform): past the last filter row; the reads are still issued, at row 0, so
        // that every trip of the loop has the same number of LDS reads in flight
        auto fetch_row = [&](RowFrags& f, int r, bool real) {
            const int rr = real ? r : 0;
            const unsigned char* ap = As + a_row + rr * (ST * 2) * APB;
#pragma unroll
            for (int t = 0; t < ST; ++t)
#pragma unroll
                for (int a = 0; a < TM; ++a) f.a[t][a] = *reinterpret_cast<const bf16x8*>(ap + t * 2 * APB + a * 32 * 16);
            // q.pw is a multiple of four positions: a filter row further is q.pw / 4 packets further in
            // the same plane (uniform), whatever the element
            const unsigned char* prow = patch + (MINUS ? -rr : rr) * (q.pw * 4);
#pragma unroll
            for (int j = 0; j < NWIN; ++j) f.w[j] = *reinterpret_cast<const bf16x8*>(prow + woff[j]);
        };
        auto multiply_row = [&](const RowFrags& f) {
#pragma unroll
            for (int t = 0; t < ST; ++t)
#pragma unroll
                for (int a = 0; a < TM; ++a)
#pragma unroll
                    for (int b = 0; b < TN; ++b)
                        acc[a][b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f.a[t][a], f.w[MINUS ? b - t + ST - 1 : b + t],
                                                                            acc[a][b], 0, 0, 0);
        };
        RowFrags f0, f1;
        fetch_row(f0, 0, true);
        int r = 0;
        // The next row's address arithmetic and LDS reads are spread between the current row's MFMAs (an
        // MFMA occupies the pipe for eight issue slots; issued in one block ahead of them, the reads
        // leave the pipe idle meanwhile, and this role has one wavefront per SIMD).
        auto spread = [&]() {
#pragma unroll
            for (int i = 0; i < ST * TM + NWIN; ++i) {
                __builtin_amdgcn_sched_group_barrier(0x008, (ST * TM * TN) / (ST * TM + NWIN), 0);   // MFMA
                __builtin_amdgcn_sched_group_barrier(0x002, 1, 0);                                  // VALU
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);                                  // LDS read
            }
            __builtin_amdgcn_sched_barrier(0);
        };
        for (; r + 2 <= p.Rt; r += 2) {
            fetch_row(f1, r + 1, true);
            multiply_row(f0);
            spread();
            fetch_row(f0, r + 2, r + 2 < p.Rt);
            multiply_row(f1);
            spread();
        }
        if (r < p.Rt) multiply_row(f0);

        group += 1;
        if (group == n_groups) {
            group = 0; tl += 1;
            const int pix_first = pix0 + wn * TN * 32 + TN * (lane & 31);
            if constexpr (!D2S) {
                store_adjacent<FUSED, TM, TN, !MINUS>(p, acc, i0, n, pix_first, pix_end, lane, bias_s + i0, i0);   // q.wv == p.Wo here
            } else {
                // this lane's coarse pixels (ho, wo .. wo + 3) in rows of q.wv: those inside the folded row
                const int ho = fastdiv(pix_first, q.div_wv);
                const int wo = pix_first - ho * q.wv;
                int hq_of[TN], wq_of[TN];
                bool live_of[TN];
#pragma unroll
                for (int b = 0; b < TN; ++b) { hq_of[b] = ho; wq_of[b] = wo + b; live_of[b] = pix_first < pix_end && wo + b < p.Wo; }
                store_d2s2_adjacent<FUSED, TM, TN>(p, acc, i0, n, hq_of, wq_of, live_of, lane);
            }
        }
    }
}

// Filter copy for the kernel above: A[group][tap][i_pad][16] with
//   mode 0 (forward)        : tap = (r, s),   ci = c, i = k
//   mode 1 (bwd, stride 1)  : tap = (r, s),   ci = k, i = c
//   mode 2 (bwd, strided)   : tap = (r', s'), ci = k, i = (c, a, b) -> w[k, c, a + sh*r', b + sw*s']
// zero beyond the last row / channel and for folded taps that fall outside the filter.
struct GroupRepack {
    const uint16_t* w; uint16_t* a;
    int mode, K, C, R, S, sh, sw, St, n_taps, Ci, Co, i_pad, total;
};
__global__ __launch_bounds__(256) void repack_groups_kernel(const GroupRepack g) {
    for (int o = blockIdx.x * 256 + threadIdx.x; o < g.total; o += gridDim.x * 256) {
        const int cl = o & (GC - 1);
        int t = o >> 4;
        const int i = t % g.i_pad;
        t /= g.i_pad;
        const int tap = t % g.n_taps;
        const int ci = (t / g.n_taps) * GC + cl;
        const int tr = tap / g.St, ts = tap - tr * g.St;
        uint16_t v = 0;
        if (i < g.Co && ci < g.Ci) {
            int k, c, r, s;
            if (g.mode == 0) { k = i; c = ci; r = tr; s = ts; }
            else if (g.mode == 1) { k = ci; c = i; r = tr; s = ts; }
            else {
                const int ph = g.sh * g.sw;
                c = i / ph;
                const int ab = i - c * ph;
                const int pa = ab / g.sw, pb = ab - pa * g.sw;
                k = ci; r = pa + g.sh * tr; s = pb + g.sw * ts;
            }
            if (r < g.R && s < g.S) v = g.w[((k * g.C + c) * g.R + r) * g.S + s];
        }
        g.a[o] = v;
    }
}

template <bool MINUS, bool D2S, bool FUSED, int TM, int ST, int ROUNDS>
hipError_t launch_roles(const PixParams& p, const PatchGeom& q, hipStream_t st) {
    auto kern = igemm_patch_roles_bf16_kernel<MINUS, D2S, FUSED, TM, ST, ROUNDS>;
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, q.roles_lds);
    if (e != hipSuccess) return e;
    ProbeScope probe(st);
    (void)hipGetLastError();
    hipLaunchKernelGGL(kern, dim3(256), dim3(512), (size_t)q.roles_lds, st, p, q);
    return hipGetLastError();
}
template <bool MINUS, bool D2S, bool FUSED>
hipError_t roles_by_shape(const PixParams& p, const PatchGeom& q, hipStream_t st) {
#define ROLES_CALL(TM, ST) (q.rounds == 1 ? launch_roles<MINUS, D2S, FUSED, TM, ST, 1>(p, q, st) \
                                          : launch_roles<MINUS, D2S, FUSED, TM, ST, 2>(p, q, st))
    switch (q.bm * 10 + p.St) {
        case 323: return ROLES_CALL(1, 3);
        case 324: return ROLES_CALL(1, 4);
        case 643: return ROLES_CALL(2, 3);
        case 644: return ROLES_CALL(2, 4);
        default: return hipErrorInvalidValue;
    }
#undef ROLES_CALL
}

template <bool MINUS, bool D2S, bool FUSED, int TM, int TN, int WM, int WN, int ROUNDS>
hipError_t launch_one(const PixParams& p, const PatchGeom& q, hipStream_t st) {
    const long long total = (long long)p.tiles_i * p.tiles_pix;
    if (total <= 0 || total > 0x7fffffffLL) return hipErrorInvalidValue;
    auto kern = igemm_patch_bf16_kernel<MINUS, D2S, FUSED, TM, TN, WM, WN, ROUNDS>;
    if (q.lds_bytes > 64 * 1024) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)q.lds_bytes);
        if (e != hipSuccess) return e;
    }
    ProbeScope probe(st);
    (void)hipGetLastError();   // drop stale status left by earlier, unrelated runtime calls
    hipLaunchKernelGGL(kern, dim3((unsigned)total), dim3(256), (size_t)q.lds_bytes, st, p, q);
    return hipGetLastError();
}

template <bool MINUS, bool D2S, bool FUSED>
hipError_t by_tile(const PixParams& p, const PatchGeom& q, hipStream_t st) {
#define PATCH_CALL(TM, TN, WM, WN)                                                     \
    (q.rounds == 1 ? launch_one<MINUS, D2S, FUSED, TM, TN, WM, WN, 1>(p, q, st)          \
                   : launch_one<MINUS, D2S, FUSED, TM, TN, WM, WN, 2>(p, q, st))
    switch (q.bm * 1000 + q.bn) {
        case 128128: return PATCH_CALL(2, 2, 2, 2);
        case 96256:  return PATCH_CALL(3, 2, 1, 4);
        case 64256:  return PATCH_CALL(2, 2, 1, 4);
        case 32256:  return PATCH_CALL(1, 2, 1, 4);
        default: return hipErrorInvalidValue;
    }
#undef PATCH_CALL
}

template <bool MINUS, bool D2S>
hipError_t by_epilogue(const PixParams& p, const PatchGeom& q, hipStream_t st) {
    const bool fused = p.bias || p.relu || p.mask;
    if (q.roles) return fused ? roles_by_shape<MINUS, D2S, true>(p, q, st) : roles_by_shape<MINUS, D2S, false>(p, q, st);
    return fused ? by_tile<MINUS, D2S, true>(p, q, st) : by_tile<MINUS, D2S, false>(p, q, st);
}

}  // namespace

namespace {
// The two-role kernel takes layers with filter rows of 3 or 4 taps whose taps all fit one stage, whose
// output rows are whole groups of four pixels (a lane's four pixels never straddle two rows) and, for
// NCHW outputs, whose rows can be written as 8-byte packets; enough tiles to keep every CU's one
// workgroup busy for several of them; two stage buffers within 156 KB of LDS. Tiles: 64 or 32 rows
// x 512 pixels. On success q and p's tile fields describe that kernel's launch.
void plan_roles(PixParams& p, int mode, PatchGeom& q) {
    if (patch_split_roles_disabled()) return;
    if (p.St != 3 && p.St != 4) return;
    if (mode != 2 && ((p.Wo & 3) || (p.out_ns & 3) || (((uintptr_t)p.out | (uintptr_t)p.mask) & 7u) != 0)) return;
    if (mode != 2 && (long long)p.Co * p.HoWo * 2 >= 0x7fffffffLL) return;   // its epilogue addresses one image as a raw buffer
    if (mode == 2 && !(p.sh == 2 && p.sw == 2 && q.d2s_buffers)) return;      // depth-to-space: the stride-2 raw-buffer epilogue only
    PatchGeom r = q;
    // patch rows of a whole number of position quads: a window element then lies in the same plane
    // (position mod 4) in every filter row, and its address moves by a constant from row to row
    r.pw = (q.pw + 3) / 4 * 4;
    r.pos_add = mode != 0 ? (p.Rt - 1) * r.pw + (p.St - 1) : 0;
    r.wv = (p.Wo + 3) / 4 * 4;
    r.div_wv = make_fastdiv(r.wv);
    r.bm = p.Co <= 32 ? 32 : 64;
    r.bn = 512;
    const int n_taps = p.Rt * p.St;
    const int rows_spanned = (r.bn - 2) / r.wv + 2;
    r.pr_max = (rows_spanned < p.Ho ? rows_spanned : p.Ho) + p.Rt - 1;
    const long long tasks = (long long)r.pr_max * r.tasks_per_row;
    if (tasks > 2 * 256) return;
    r.rounds = tasks > 256 ? 2 : 1;
    // (+ 4 positions: the windows of the pixels past a row's end run past the last patch row)
    const long long plane = ((long long)r.pr_max * r.pw + 4 + 3) / 4 * 16;
    r.plane_bytes = (int)((plane + 95) / 128 * 128 + 32);      // 32 past a multiple of 128
    const long long a_tap = 2LL * (r.bm * 16 + 64);
    if ((long long)n_taps * r.bm * 2 > (long long)A_ROUNDS * 256) return;
    r.taps_per_stage = n_taps;
    r.a_rounds = (int)(((long long)n_taps * r.bm * 2 + 255) / 256);
    r.a_bytes = (int)(n_taps * a_tap);
    r.tiles_per_img = (p.Ho * r.wv + r.bn - 1) / r.bn;
    const long long tiles_pix = (long long)p.N * r.tiles_per_img;
    const int tiles_i = (p.Co + r.bm - 1) / r.bm;
    if (tiles_pix * tiles_i > 0x7fffffffLL) return;
    if (tiles_pix * tiles_i < 4 * 256 && !patch_split_roles_forced()) return;
    const long long i_pad = (long long)tiles_i * r.bm;
    const long long lds = i_pad * 4 + 2LL * (r.a_bytes + 2LL * RTN * r.plane_bytes + 128);
    if (lds > 156 * 1024) return;
    if ((long long)n_taps * i_pad * p.Ci_pad > 0x7fffffffLL) return;
    r.div_tpi = make_fastdiv(r.tiles_per_img);
    r.roles = 1;
    r.roles_lds = (int)lds;
    r.pairs = 1;
    q = r;
    p.tiles_i = tiles_i;
    p.tiles_pix = (int)tiles_pix;
    p.i_pad = (int)i_pad;
}
}  // namespace

// p: the pass's geometry as the tap-major kernel gets it (Ci, Co, Rt, St, gather origin, extents).
// On success p.Ci_pad / p.i_pad / p.tiles_i / p.tiles_pix / p.in_bytes describe this kernel's launch
// and q its patch; the caller repacks the filter (repack_patch_filter) into scratch of at least
// patch_filter_bytes and launches. mode: 0 forward, 1 backward-data unit stride, 2 phase-folded.
bool plan_patch_bf16(PixParams& p, int mode, PatchGeom* qg) {
    const bool minus = mode != 0;
    if (p.g_mul_h != 1 || p.g_mul_w != 1) return false;
    if ((p.Wi & 7) || (p.in_ns & 7) || (p.Ci & 7)) return false;
    if ((((uintptr_t)p.in) & 15u) != 0) return false;
    const long long in_bytes = ((long long)(p.N - 1) * p.in_ns + (long long)p.Ci * p.HiWi) * 2;
    if (in_bytes >= 0x7fffffffLL) return false;
    // row tile: least padded channel count, the larger tile on ties
    const int cand[4][2] = {{128, 128}, {96, 256}, {64, 256}, {32, 256}};
    PatchGeom q{};
    long long best = -1;
    for (const auto& c : cand) {
        const long long padded = (long long)((p.Co + c[0] - 1) / c[0]) * c[0];
        if (best < 0 || padded < best) { best = padded; q.bm = c[0]; q.bn = c[1]; }
    }
    const int n_taps = p.Rt * p.St;
    q.pw = p.Wo + p.St - 1;                                   // patch columns (one spare column may follow on the right)
    const int rows_spanned = (q.bn - 2) / p.Wo + 2;
    q.pr_max = (rows_spanned < p.Ho ? rows_spanned : p.Ho) + p.Rt - 1;
    q.w_lo = p.g_add_w - (minus ? p.St - 1 : 0);
    q.h_lo_add = p.g_add_h - (minus ? p.Rt - 1 : 0);
    q.pos_add = minus ? (p.Rt - 1) * q.pw + (p.St - 1) : 0;
    q.chunks = p.Wi / 8;
    q.halo_l = -q.w_lo;
    q.halo_r0 = p.Wi - q.w_lo;
    if (q.halo_l < 0 || q.halo_r0 > q.pw) return false;       // image columns outside the patch
    q.tasks_per_row = (q.chunks + 3) / 4 * 4 * (GC / 8);
    const long long tasks = (long long)q.pr_max * q.tasks_per_row;
    if (tasks > 2 * 256) return false;
    q.rounds = tasks > 256 ? 2 : 1;
    // taps per stage: as many as the thread's filter registers and 80 KB of LDS (two workgroups per
    // CU) allow; whole filter rows when a stage cannot hold every tap
    const long long plane = ((long long)q.pr_max * q.pw + 1) / 2 * 16;
    q.plane_bytes = (int)((plane + 95) / 128 * 128 + 32);      // 32 past a multiple of 128
    const long long patch_bytes = 4LL * q.plane_bytes + 128;    // + spare packets for threads without a task
    const long long fixed = (long long)q.bm * 4 + patch_bytes;
    const long long a_tap = 2LL * (q.bm * 16 + 64);            // LDS bytes of one tap's filter rows
    long long tc = (long long)A_ROUNDS * 256 / (q.bm * 2);
    const long long by_lds = (80 * 1024 - fixed) / a_tap;
    if (by_lds < tc) tc = by_lds;
    if (tc > n_taps) tc = n_taps;
    if (tc < 1) return false;
    if (tc < n_taps && tc > p.St) tc = tc / p.St * p.St;
    q.taps_per_stage = (int)tc;
    q.a_rounds = (int)((tc * q.bm * 2 + 255) / 256);
    q.a_bytes = (int)(tc * a_tap);
    q.lds_bytes = (int)(fixed + q.a_bytes);
    q.tiles_per_img = (p.HoWo + q.bn - 1) / q.bn;
    q.div_tpi = make_fastdiv(q.tiles_per_img);
    q.div_tpr = make_fastdiv(q.tasks_per_row);
    q.div_chunks = make_fastdiv(q.chunks);
    q.div_st = make_fastdiv(p.St);
    const int halo_w = q.halo_l + q.pw - q.halo_r0;
    q.div_halo = make_fastdiv(halo_w > 0 ? halo_w : 1);
    const long long tiles_pix = (long long)p.N * q.tiles_per_img;
    if (tiles_pix > 0x7fffffffLL) return false;
    p.tiles_i = (p.Co + q.bm - 1) / q.bm;
    p.tiles_pix = (int)tiles_pix;
    p.i_pad = p.tiles_i * q.bm;
    p.Ci_pad = (p.Ci + GC - 1) / GC * GC;
    if ((long long)n_taps * p.i_pad * p.Ci_pad > 0x7fffffffLL) return false;
    p.in_bytes = (unsigned)in_bytes;
    // 4-byte stores of pixel pairs: every row of every image starts at an even element
    // (the paired epilogue addresses one image of the output as a raw buffer: below 2^31 bytes)
    q.pairs = ((p.HoWo | p.out_ns) & 1) == 0 && (((uintptr_t)p.out | (uintptr_t)p.mask) & 3u) == 0 &&
              (long long)p.Co * p.HoWo * 2 < 0x7fffffffLL;
    // depth-to-space outputs through raw buffer stores: one image of dx below 2^31 bytes
    q.d2s_buffers = mode == 2 && (long long)p.C * p.H * p.W * 2 < 0x7fffffffLL && !buffer_loads_disabled();
    q.roles = 0;
    plan_roles(p, mode, q);       // the two-role kernel where it applies: replaces tile, patch and stage geometry
    *qg = q;
    return true;
}

// bytes of the repacked filter for a layer with Co output rows, Ci gathered channels and n_taps taps,
// whatever row tile ends up running
size_t patch_filter_bytes(int Co, int Ci, int n_taps) {
    const long long i_pad = ((long long)Co + 127) / 128 * 128;   // the row tile picked never pads further than 128-row tiles
    return (size_t)n_taps * (size_t)i_pad * (size_t)((Ci + GC - 1) / GC * GC) * 2;
}

hipError_t repack_patch_filter(const PixParams& p, int mode, const void* w, void* a, int K, int C, hipStream_t st) {
    GroupRepack g{};
    g.w = (const uint16_t*)w; g.a = (uint16_t*)a;
    g.mode = mode; g.K = K; g.C = C; g.R = p.R; g.S = p.S; g.sh = p.sh; g.sw = p.sw;
    g.St = p.St; g.n_taps = p.Rt * p.St; g.Ci = p.Ci; g.Co = p.Co; g.i_pad = p.i_pad;
    g.total = g.n_taps * p.i_pad * p.Ci_pad;
    const long long blocks = ((long long)g.total + 255) / 256;
    (void)hipGetLastError();
    hipLaunchKernelGGL(repack_groups_kernel, dim3((unsigned)(blocks > 4096 ? 4096 : blocks)), dim3(256), 0, st, g);
    return hipGetLastError();
}

hipError_t launch_patch_bf16(const PixParams& p, const PatchGeom& q, int mode, hipStream_t st) {
    if (mode == 0) return by_epilogue<false, false>(p, q, st);
    if (mode == 1) return by_epilogue<true, false>(p, q, st);
    return by_epilogue<true, true>(p, q, st);
}

}  // namespace pix
}  // namespace purine

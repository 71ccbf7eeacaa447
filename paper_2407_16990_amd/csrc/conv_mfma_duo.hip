// 64 -> 64-channel-chunk bf16 conv3x3 on the matrix cores, two-team variant.
//
// Same implicit GEMM, LDS layouts, fragment order and buffer addressing as k_conv_mfma
// (conv_mfma.hip), but the workgroup has 8 waves = two teams of 4.  The teams share the
// LDS-resident weights and own one 10 x 34 pixel patch each: a team computes one half (8 x 32
// pixels) of a 16 x 32 tile at a time.  The teams run one half apart: while one team is in its
// MFMA loop, the other rounds its finished accumulators to bf16, adds the skip tensor, writes
// the result, and puts its next patch into LDS.  Every SIMD holds one wave of each team, so the
// matrix pipe is fed by one wave while the other does vector-ALU, LDS and memory work.
//
// The hardware barrier counts all 8 waves, so both teams execute the same barrier sequence:
// time is cut into phases of exactly two barriers.
//   compute phase : MFMA steps 0..MID-1 | barrier | steps MID..11 | barrier
//                   (LDS fragment reads and MFMAs only: a wave that issues a wide global memory
//                   instruction cannot issue MFMAs for some 60-90 cycles, so the MFMA loop
//                   carries none)
//   drain phase   : issue the global loads (next patch, skip), accumulators -> bf16 -> own LDS
//                   slice -> registers, + skip, global stores | barrier |
//                   next patch registers -> LDS | barrier
// Team 0 runs compute, drain, compute, ...; team 1 starts with an idle phase, so the phases
// pair up.  The unit of work is the half tile (8 x 32 pixels): the halves are numbered 2 * tile +
// half and dealt out so that workgroup w takes units w, w + G, w + 2G, ... alternately with team 0
// and team 1 (G workgroups).  When the units do not divide evenly team 1 has one unit fewer than
// team 0 and ends with the idle phase instead (a whole tile per workgroup as the unit would leave
// half the chip idle for a full round whenever the tile count is not a multiple of G).  The
// number of phases depends only on kernel arguments, the workgroup index and - with a tile list -
// the list's length (never on anything that differs between the waves of a workgroup), the
// prefetch past a team's last unit loads out of range (zeros), and no wave leaves the loop
// early: every barrier is reached by all 8 waves.
#include <stdlib.h>

#include <type_traits>

#include "conv_mfma_common.h"

#define PW 34
template <int N, int I = 0, typename F>
__device__ __forceinline__ void for_each_step2(F& f)
{
    if constexpr (I < N) { f(std::integral_constant<int, I>{}); for_each_step2<N, I + 1>(f); }
}

__device__ __forceinline__ void phase_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }
__device__ __forceinline__ void idle_phase() { phase_barrier(); phase_barrier(); }

// LIST: the half tiles to compute come from a.tile_list (box-masked mode) instead of being all of
// all images.  The entry of the next tile is requested with a vector load at the start of the
// compute phase and read at the start of the drain phase, a whole phase later: a scalar load would
// share its counter with the LDS fragment reads and turn their partial waits into full ones.
template <bool SKIP, bool RELU, int MID, bool LIST>
__global__ __launch_bounds__(512) void k_conv_mfma_duo(conv_args a)
{
    constexpr int CIN = 64, MT = 2, KS = 4, NCH = 8, PIXB = 128, TH = 8, PH = TH + 2, RW = 2, NR = RW + 2;
    constexpr int WBYTES = 9 * KS * MT * 1024, PATCHB = PH * PW * PIXB, NSTEP = 3 * KS, CQ = 64;
    constexpr int NMAIN = PH, NHP = PH * 2 * NCH, NHALO = 1, NPRE = NMAIN + NHALO;      // 16-byte patch pieces per thread
    static_assert(NHP <= 256, "halo pieces must fit one per thread");
    // The accumulators start from the bias.  The skip variant's drain phase is the longer of the two
    // phases, so there the seeding belongs to the compute phase; otherwise it is done in the drain phase.
    constexpr bool SEED_IN_COMPUTE = SKIP;
    constexpr bool SKIP_IN_COMPUTE = true;
    static_assert(MID >= 1 && MID <= NSTEP - 1, "the compute phase must hold exactly two barriers");
    // MID: the compute phase's first barrier comes after MID of the 12 steps; it pairs with the end
    // of the other team's loads + rounding + skip add + stores
    constexpr int NCHO = 8, OPIXB = 128, NOUT = RW * 32 * NCHO / 64, PPJ = 8, JPR = 4;   // output pieces per lane

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    // team and wave are uniform over a wave: taken through readfirstlane so that the compiler keeps
    // everything derived from them (tile rows, row validity, descriptors) in scalar registers
    const int tid = threadIdx.x, ttid = tid & 255, lane = tid & 63;
    const int team = __builtin_amdgcn_readfirstlane(tid >> 8), wave = __builtin_amdgcn_readfirstlane((tid >> 6) & 3);
    const int lx = lane & 31, hi = lane >> 5;
    uint8_t* lds_w = lds;
    uint8_t* lds_p = lds + WBYTES + team * PATCHB;
    float* lds_b = (float*)(lds + WBYTES + 2 * PATCHB);       // the chunk's 64 biases

    const int n_img = a.n_valid ? min((int)*a.n_valid, a.N) : a.N;
    const int tiles_x = (a.W + 31) / 32, tiles_y = (a.H + 15) / 16;
    const int tiles_img = tiles_x * tiles_y;
    // half tiles; with a list, its entries are half tiles packed as RH_CELL_ENTRY(image, row of 8, column of 32)
    const int n_units = LIST ? (int)*a.n_list : 2 * n_img * tiles_img;
    // Tile order.  Workgroups go to the 8 XCDs round-robin; XCD x takes a contiguous run of tile
    // lanes so that neighbouring tiles (shared halo pixels) meet in one L2.
    // Layers with several output chunks (the upsampling convs): when the grid allows it the chunks
    // are dealt to workgroups instead of looped over - the n_chunks workgroups of one XCD that
    // share a tile lane process the same tiles at about the same time, each with its own chunk's
    // weights resident, so the input is fetched from HBM once and the other reads hit L2
    // (looping chunks outermost reads the whole input once per chunk).
    const bool deal = a.n_chunks > 1 && gridDim.x % (8 * a.n_chunks) == 0;
    const int G = deal ? gridDim.x / a.n_chunks : gridDim.x;                  // tile lanes
    const int xcd = blockIdx.x % 8, local = blockIdx.x / 8;
    const int wg = deal ? xcd * (G / 8) + local / a.n_chunks
                        : ((G % 8 == 0) ? xcd * (G / 8) + local : (int)blockIdx.x);
    const int chunk_begin = deal ? local % a.n_chunks : 0, chunk_end = deal ? chunk_begin + 1 : a.n_chunks;
    auto units_from = [&](int first) { return n_units > first ? (n_units - first + 2 * G - 1) / (2 * G) : 0; };
    const int u_first = wg + team * G;                         // this team's units: u_first, u_first + 2G, ...
    const int iters0 = units_from(wg), iters1 = units_from(wg + G);           // team 1 has as many as team 0 or one fewer
    const int iters = team ? iters1 : iters0;
    const int ps = a.ps;
    const uint32_t in_img_bytes = (uint32_t)a.H * a.W * PIXB;
    const uint32_t out_img_bytes = (uint32_t)(a.H * ps) * (a.W * ps) * OPIXB;

    // per-thread constants of the patch pieces (see k_conv_mfma)
    const int m_col = ttid >> 3, m_c = ttid & 7;
    const int m_goff = m_col * PIXB + m_c * 16;
    const uint32_t m_lds = (uint32_t)((1 + m_col) * PIXB + ((m_c ^ ((1 + m_col) & 7)) << 4));
    const int h_row = ttid >> 4, h_side = (ttid >> 3) & 1, h_c = ttid & 7;     // halo piece (ttid < NHP)
    const int lcol = lane >> 3, lc = lane & 7;
    const int o_lane = (lcol * ps) * OPIXB + lc * 16;
    const int o_rowpitch = a.W * ps * OPIXB;
    const int row_pitch = a.W * PIXB;

    // origin of half `half` of tile number `tile` (rows y0..y0+7), image index n
    auto decode = [&](int tile, int half, int& n, int& y0, int& x0) __attribute__((always_inline)) {
        n = tile / tiles_img;
        const int tr = tile - n * tiles_img, ty = tr / tiles_x, tx = tr - ty * tiles_x;
        y0 = ty * 16 + half * TH; x0 = tx * 32;
    };
    // Consecutive layers walk the tensor in opposite directions: what a layer touched last (the
    // end of its input and output) is what the next layer touches first, while it is still in
    // the memory-side cache.  Walking every layer front to back through buffers that together
    // exceed that cache evicts each line just before it is needed again.
    __amdgpu_buffer_rsrc_t rlist = __builtin_amdgcn_make_buffer_rsrc((void*)a.tile_list, 0, LIST ? (uint32_t)n_units * 4u : 0u, RSRC_FLAGS);
    auto walk = [&](int u) __attribute__((always_inline)) { return (a.rev && u < n_units) ? n_units - 1 - u : u; };
    auto list_load = [&](int u) __attribute__((always_inline)) {         // list entry of unit u (0 past the end)
        return __builtin_amdgcn_raw_buffer_load_b32(rlist, u < n_units ? (uint32_t)walk(u) * 4u : OOB_OFF, 0, 0);
    };
    auto decode_cell = [&](int cell, int& n, int& y0, int& x0) __attribute__((always_inline)) {
        n = (int)((uint32_t)cell >> 16); y0 = (int)(((uint32_t)cell >> 7) & 511u) * TH; x0 = (int)((uint32_t)cell & 127u) * 32;
    };
    auto unit_origin = [&](int u, int& n, int& y0, int& x0) __attribute__((always_inline)) {
        if constexpr (LIST) decode_cell(__builtin_amdgcn_readfirstlane(list_load(u)), n, y0, x0);
        else { const int uu = walk(u); decode(uu >> 1, uu & 1, n, y0, x0); }
    };
    uint4 pre[NPRE];
    auto load_piece = [&](int j, __amdgpu_buffer_rsrc_t rin, int y0, int x0) __attribute__((always_inline)) {
        int off; bool ok;
        if (j < NMAIN) {
            const int gy = y0 - 1 + j;
            ok = gy >= 0 && gy < a.H && x0 + m_col < a.W;
            off = ((y0 - 1) * a.W + x0) * PIXB + m_goff + j * row_pitch;
        } else {
            const int gy = y0 - 1 + h_row, hx = h_side ? x0 + 32 : x0 - 1;
            ok = ttid < NHP && gy >= 0 && gy < a.H && hx >= 0 && hx < a.W;
            off = (gy * a.W + hx) * PIXB + h_c * 16;
        }
        const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rin, ok ? (uint32_t)off : OOB_OFF, 0, 0);
        pre[j] = make_uint4(v[0], v[1], v[2], v[3]);
    };
    auto store_patch = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NMAIN; ++j) *(uint4*)(lds_p + j * (PW * PIXB) + m_lds) = pre[j];
        const int px = h_side ? PW - 1 : 0;
        if (ttid < NHP) *(uint4*)(lds_p + (h_row * PW + px) * PIXB + ((h_c ^ (px & 7)) << 4)) = pre[NMAIN];
    };
    auto out_off = [&](int j, int y0, int x0, int si, int sj) __attribute__((always_inline)) {
        const int y = y0 + wave * RW + j / JPR, xb = x0 + (j % JPR) * PPJ;
        const bool ok = y < a.H && xb + lcol < a.W;
        const int off = (y * ps + si) * o_rowpitch + (xb * ps + sj) * OPIXB + o_lane;
        return ok ? (uint32_t)off : OOB_OFF;
    };
    auto in_rsrc = [&](int u, int n) __attribute__((always_inline)) {
        return __builtin_amdgcn_make_buffer_rsrc((void*)(a.in + (size_t)n * a.H * a.W * CIN), 0,
                                                 u < n_units ? in_img_bytes : 0u, RSRC_FLAGS);
    };

    int cn = 0, cy0 = 0, cx0 = 0;                          // LIST: origin of the tile about to be computed
    for (int chunk = chunk_begin; chunk < chunk_end; ++chunk) {
        __syncthreads();                                   // all 8 waves: previous chunk completely done
        {   // the chunk's weights and the first patch of both teams: all loads are issued before
            // the first LDS store waits for any of them
            constexpr int NWL = WBYTES / 16 / 512;         // 16-byte weight pieces per thread
            static_assert(NWL * 512 * 16 == WBYTES, "weights must split evenly over the workgroup");
            const uint4* src = a.wp + (size_t)chunk * (WBYTES / 16);
            int n, y0, x0; unit_origin(u_first, n, y0, x0);
            cn = n; cy0 = y0; cx0 = x0;
            __amdgpu_buffer_rsrc_t rin = in_rsrc(u_first, u_first < n_units ? n : 0);
#pragma unroll
            for (int j = 0; j < NPRE; ++j) load_piece(j, rin, y0, x0);
            constexpr int WB = 3;                          // weight pieces in flight per thread (register budget)
#pragma unroll
            for (int i0 = 0; i0 < NWL; i0 += WB) {
                uint4 wreg[WB];
#pragma unroll
                for (int i = 0; i < WB; ++i) if (i0 + i < NWL) wreg[i] = src[(i0 + i) * 512 + tid];
#pragma unroll
                for (int i = 0; i < WB; ++i) if (i0 + i < NWL) ((uint4*)lds_w)[(i0 + i) * 512 + tid] = wreg[i];
            }
            if (tid < CQ) lds_b[tid] = a.bias[chunk * CQ + tid];
            store_patch();
        }
        const int si = chunk / ps, sj = chunk - si * ps;
        __syncthreads();

        // accumulators start from the bias: lane holds channels m*32 + 8*q + 4*hi + {0..3} in
        // acc[.][m][4q..4q+3].  They are re-seeded in the drain phase, off the critical path.
        f32x16 acc[RW][MT];
        auto seed_acc = [&]() __attribute__((always_inline)) {
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const float4 bv = *(const float4*)(lds_b + m * 32 + q * 8 + hi * 4);
#pragma unroll
                    for (int r = 0; r < RW; ++r) { acc[r][m][4 * q] = bv.x; acc[r][m][4 * q + 1] = bv.y; acc[r][m][4 * q + 2] = bv.z; acc[r][m][4 * q + 3] = bv.w; }
                }
        };
        if constexpr (!SEED_IN_COMPUTE) seed_acc();
        if (team == 1) idle_phase();
        for (int it = 0; it < iters; ++it) {
            const int unit = u_first + it * 2 * G, nunit = unit + 2 * G;
            int n, y0, x0, next_entry = 0;
            if constexpr (LIST) { n = cn; y0 = cy0; x0 = cx0; next_entry = list_load(nunit); }
            else unit_origin(unit, n, y0, x0);
            __amdgpu_buffer_rsrc_t rsk = __builtin_amdgcn_make_buffer_rsrc(
                (void*)((uint8_t*)a.skip + (size_t)n * out_img_bytes), 0, SKIP ? out_img_bytes : 0u, RSRC_FLAGS);
            uint4 sk[SKIP ? NOUT : 1];
            // ---------------- compute phase ----------------
            if constexpr (SEED_IN_COMPUTE) seed_acc();
            const uint8_t* wlane = lds_w + (lane << 4);
            const uint8_t* prow = lds_p + (wave * RW) * (PW * PIXB);
            bf16x8 A0[3][MT], A1[3][MT], B0[NR], B1[NR];
            {   // fragments of step 0
                const uint8_t* b0 = prow + lx * PIXB + ((hi ^ (lx & 7)) << 4);
#pragma unroll
                for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                    for (int m = 0; m < MT; ++m) A0[ky][m] = *(const bf16x8*)(wlane + ((((ky * 3) * KS) * MT + m) << 10));
#pragma unroll
                for (int py = 0; py < NR; ++py) B0[py] = *(const bf16x8*)(b0 + py * (PW * PIXB));
            }
            auto step = [&](auto st_c) __attribute__((always_inline)) {
                constexpr int st = decltype(st_c)::value;
                constexpr int NMF = 3 * RW * MT, NFR = 3 * MT + NR, NSLOT = 6;
                constexpr int MPS = NMF / NSLOT, FPS = (NFR + NSLOT - 1) / NSLOT;
                bf16x8 (&Ac)[3][MT] = (st & 1) ? A1 : A0;
                bf16x8 (&Bc)[NR] = (st & 1) ? B1 : B0;
                bf16x8 (&An)[3][MT] = (st & 1) ? A0 : A1;
                bf16x8 (&Bn)[NR] = (st & 1) ? B0 : B1;
                constexpr int kxn = (st + 1) / KS, ksn = (st + 1) - kxn * KS;
                const int pxn = lx + kxn;
                const uint8_t* b0n = prow + pxn * PIXB + (((2 * ksn + hi) ^ (pxn & 7)) << 4);
#pragma unroll
                for (int sl = 0; sl < NSLOT; ++sl) {
                    if (st + 1 < NSTEP) {
#pragma unroll
                        for (int f = sl * FPS; f < (sl + 1) * FPS && f < NFR; ++f) {
                            // fragments in the order of their first use in the next step:
                            // B0, A0*, B1, A1*, B2, A2*, B3  (A ky-th pair follows B ky)
                            constexpr int GRP = 1 + MT;
                            const int g = f / GRP, w = f % GRP;
                            if (g < 3 && w > 0) An[g][w - 1] = *(const bf16x8*)(wlane + ((((g * 3 + kxn) * KS + ksn) * MT + (w - 1)) << 10));
                            else Bn[g < 3 ? g : 3 + (f - 3 * GRP)] = *(const bf16x8*)(b0n + (g < 3 ? g : 3 + (f - 3 * GRP)) * (PW * PIXB));
                        }
                    }
#pragma unroll
                    for (int k = sl * MPS; k < (sl + 1) * MPS; ++k) {
                        const int m = k % MT, pair = k / MT;
                        int py = 0, ky = 0, cnt = 0;
#pragma unroll
                        for (int p = 0; p < NR; ++p)
#pragma unroll
                            for (int q = 0; q < 3; ++q)
                                if (p - q >= 0 && p - q < RW) { if (cnt == pair) { py = p; ky = q; } ++cnt; }
                        const int r = py - ky;
                        acc[r][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ac[ky][m], Bc[py], acc[r][m], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (SKIP && SKIP_IN_COMPUTE && st < NOUT) {
                    const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsk, out_off(st, y0, x0, 0, 0), 0, 0);
                    sk[st] = make_uint4(v[0], v[1], v[2], v[3]);
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (LIST && st == MID - 1) {              // the next unit's list entry has long arrived: decode it here,
                    decode_cell(__builtin_amdgcn_readfirstlane(next_entry), cn, cy0, cx0);   // off the drain phase's critical path
                    __builtin_amdgcn_sched_barrier(0);
                }
                if constexpr (st == MID - 1 || st == NSTEP - 1) {   // the two barriers of the compute phase
                    asm volatile("s_barrier" ::: "memory");
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            __builtin_amdgcn_s_setprio(2);             // the wave feeding the matrix pipe goes first
            for_each_step2<NSTEP>(step);
            __builtin_amdgcn_s_setprio(0);

            // ---------------- drain phase ----------------
            int nn, ny0, nx0;
            if constexpr (LIST) { nn = cn; ny0 = cy0; nx0 = cx0; }
            else unit_origin(nunit, nn, ny0, nx0);
            __amdgpu_buffer_rsrc_t rin = in_rsrc(nunit, nunit < n_units ? nn : 0);
            __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
                (void*)((uint8_t*)a.out + (size_t)n * out_img_bytes), 0, out_img_bytes, RSRC_FLAGS);
            // The global loads of the next tile's patch (stored to LDS at the end of the phase) are
            // issued here, by waves that are not feeding the matrix pipe.  The skip variant's
            // drain phase is the longer of the two phases: there the tile's skip values are loaded
            // during its own compute phase instead (one load after each of the first 8 steps), which
            // costs the matrix pipe a few issue slots but takes their issue time and their whole
            // latency off the critical phase.  The CU's one address unit
            // takes about 16 cycles per 64 x 16-byte instruction and all four waves of the team
            // arrive together, so a wave that issues its loads back to back is held for 60-90
            // cycles by each of them: the loads are dealt out one or two at a time between the
            // 16 units of rounding work instead.
            constexpr bool SKIP_HERE = SKIP && !SKIP_IN_COMPUTE;
            constexpr int NLD = NPRE + (SKIP_HERE ? NOUT : 0), NUNIT = MT * 4 * RW;
            auto issue_load = [&](int i) __attribute__((always_inline)) {
                if (SKIP_HERE && i < NOUT) {
                    const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsk, out_off(i, y0, x0, 0, 0), 0, 0);
                    sk[i] = make_uint4(v[0], v[1], v[2], v[3]);
                } else {
                    load_piece(i - (SKIP_HERE ? NOUT : 0), rin, ny0, nx0);
                }
            };
            uint8_t* stg = lds_p + wave * (RW * 32 * OPIXB);
            const int okey = lx & 7;
#pragma unroll
            for (int m = 0; m < MT; ++m)
#pragma unroll
                for (int q = 0; q < 4; ++q)
#pragma unroll
                    for (int r = 0; r < RW; ++r) {
                        const int u = (m * 4 + q) * RW + r;
#pragma unroll
                        for (int i = u * NLD / NUNIT; i < (u + 1) * NLD / NUNIT; ++i) issue_load(i);
                        float v0 = acc[r][m][4 * q + 0], v1 = acc[r][m][4 * q + 1], v2 = acc[r][m][4 * q + 2], v3 = acc[r][m][4 * q + 3];
                        uint2 pk;
                        pk.x = pack_bf16x2(v0, v1); pk.y = pack_bf16x2(v2, v3);
                        if constexpr (RELU) { pk.x = relu_bf16x2(pk.x); pk.y = relu_bf16x2(pk.y); }   // rounding keeps the sign
                        *(uint2*)(stg + (r * 32 + lx) * OPIXB + (((m * 4 + q) ^ okey) << 4) + hi * 8) = pk;
                        __builtin_amdgcn_sched_barrier(0);
                    }
            if constexpr (!SEED_IN_COMPUTE) seed_acc();
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");     // the slice is private to the wave: no barrier
            uint4 ov[NOUT];
#pragma unroll
            for (int j = 0; j < NOUT; ++j) {
                const int r = j / JPR, px = (j % JPR) * PPJ + lcol;
                ov[j] = *(const uint4*)(stg + (r * 32 + px) * OPIXB + ((lc ^ (px & 7)) << 4));
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int j = 0; j < NOUT; ++j) {
                uint4 o = ov[j];
                if constexpr (SKIP) {
                    o.x = pack_bf16x2(bf16_lo(o.x) + bf16_lo(sk[j].x), bf16_hi(o.x) + bf16_hi(sk[j].x));
                    o.y = pack_bf16x2(bf16_lo(o.y) + bf16_lo(sk[j].y), bf16_hi(o.y) + bf16_hi(sk[j].y));
                    o.z = pack_bf16x2(bf16_lo(o.z) + bf16_lo(sk[j].z), bf16_hi(o.z) + bf16_hi(sk[j].z));
                    o.w = pack_bf16x2(bf16_lo(o.w) + bf16_lo(sk[j].w), bf16_hi(o.w) + bf16_hi(sk[j].w));
                }
                const i32x4 v = {(int)o.x, (int)o.y, (int)o.z, (int)o.w};
                __builtin_amdgcn_raw_buffer_store_b128(v, rout, out_off(j, y0, x0, si, sj), 0, 0);
                if constexpr (SKIP) __builtin_amdgcn_sched_barrier(0);
            }
            phase_barrier();                                  // 1: every wave of the team has read its slice back
            store_patch();                                    // next tile's patch (zeros after the last tile)
            phase_barrier();                                  // 2
        }
        // team 0's last drain phase pairs with team 1's last one, or - team 1 a unit short - with its idle phase
        if (team == 0 ? iters1 == iters0 : iters1 < iters0) idle_phase();
    }
}

template <bool SKIP, bool RELU, int MID, bool LIST>
static hipError_t launch_duo(hipStream_t stream, int device, const conv_args& a, int grid)
{
    constexpr int lds = 9 * 4 * 2 * 1024 + 2 * 10 * PW * 128 + 256;
    static bool attr_done[RH_MAX_DEVICES] = {};            // the attribute is per device
    if (!attr_done[device]) {
        hipError_t e = hipFuncSetAttribute((const void*)k_conv_mfma_duo<SKIP, RELU, MID, LIST>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_done[device] = true;
    }
    hipLaunchKernelGGL((k_conv_mfma_duo<SKIP, RELU, MID, LIST>), dim3(grid), dim3(512), lds, stream, a);
    return hipGetLastError();
}

hipError_t rh_launch_conv_duo(hipStream_t stream, int device, const conv_args& a, int grid, bool skip, bool relu)
{
    // first barrier of the compute phase after 10 of the 12 steps (A/B on one box: 0.7 % better than 11, 9 is worse)
    constexpr int MID = 10;
    if (a.tile_list) {
        if (a.n_chunks != 1) return hipErrorInvalidValue;      // a tile list goes with single-chunk layers only
        if (skip) return launch_duo<true, false, MID, true>(stream, device, a, grid);
        if (relu) return launch_duo<false, true, MID, true>(stream, device, a, grid);
        return launch_duo<false, false, MID, true>(stream, device, a, grid);
    }
    if (skip) return launch_duo<true, false, MID, false>(stream, device, a, grid);
    if (relu) return launch_duo<false, true, MID, false>(stream, device, a, grid);
    return launch_duo<false, false, MID, false>(stream, device, a, grid);
}

// SR forward, bf16 path (Sec. 3.3.3): every 3x3 convolution with C input channels is an
// implicit GEMM on the bf16 matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulate).
//
// GEMM view of one conv:  D[cout][pixel] = sum_k A[cout][k] * B[k][pixel],  k = tap*CIN + ci.
//   A (weights) and B (activations) both come from LDS:
//   - the workgroup is persistent and keeps one 64-output-channel chunk of the weights in
//     LDS for all the tiles it processes (repacked at rh_create into MFMA fragment order, so
//     a fragment load is one conflict-free 16-byte read per lane);
//   - per tile it stages the (TH+2) x (TW+2) halo'd activation patch, channels last, with
//     the eight 16-byte channel groups of a pixel XOR-swizzled by the pixel's column so
//     that 32 lanes reading 32 neighbouring pixels hit distinct banks.
//   Output channels sit on the M side so that a lane ends up holding 4 consecutive channels
//   of one pixel (an 8-byte channels-last store).
// Activations are bf16 channels-last [N][H][W][C]; the network's last conv writes fp32.
// Pixel shuffle is folded into the output-channel order of the upsampling convs: chunk q of
// the permuted weights produces all C channels of sub-pixel q, i.e. one whole output pixel.
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "conv_mfma_common.h"

#define TW 32            // tile width in pixels = N of one MFMA
#define PW (TW + 2)


// CIN: input channels (32 or 64).  MT: 32-channel M tiles per output chunk (1 or 2).
// TH: tile height; each of the 4 waves owns RW = TH/4 rows of 32 pixels.
// F32OUT: last layer of the network (fp32 output, true channel count cout_real <= 32*MT,
// optional pixel shuffle s_final in the store address).  SKIP: add a same-shaped bf16 tensor
// to the output (residual connections).  RELU: clamp at zero before rounding.  MINB: workgroups
// that must fit on a CU together (2 for the memory-bound last layer: small tiles, so that one
// workgroup's loads overlap the other's MFMAs; 1 = all registers and LDS for one workgroup).
//
// Per tile:   (A) barrier, prefetched patch registers -> LDS, (B) barrier, MFMA loop,
//             (C) barrier, accumulators -> bf16 -> LDS, (D) barrier, LDS -> registers.
// MFMA loop:  NSTEP = 3 * CIN/16 steps = (kx, k-step) pairs.  In a step the 3 x MT weight
//             fragments of the three ky taps stay in registers while the wave walks down its
//             RW+2 input rows: every activation fragment is read from LDS once and feeds the
//             (up to) 3 output rows it belongs to.  The fragments of step s+1 are loaded while
//             the MFMAs of step s run (two register sets).  The accumulators start from the
//             bias (C operand of the first MFMA).
// Memory:     all global traffic of a tile is issued from inside the MFMA loop, a few
//             instructions per step, so that it is never waited for while the matrix cores
//             idle: the stores of the PREVIOUS tile's result (kept in registers), the loads of
//             the NEXT tile's patch (into registers), and in the last steps the skip reads of
//             the current tile.  Buffer instructions are used: out-of-range lanes (ragged
//             tiles, the zero padding around the image, "no previous / no next tile") get an
//             offset beyond the descriptor's size, which makes loads return 0 and drops stores,
//             so there is no branch and no masking.
// Epilogue:   results go through the wave's own slice of the (then free) patch area and are
//             read back as 16-byte channel groups: the skip read and the store move whole
//             pixels, 1 KB contiguous per wave instruction.
template <int N, int I = 0, typename F>
__device__ __forceinline__ void for_each_step(F& f)
{
    if constexpr (I < N) { f(std::integral_constant<int, I>{}); for_each_step<N, I + 1>(f); }
}


template <int CIN, int MT, int TH, bool F32OUT, bool SKIP, bool RELU, int MINB>
__global__ __launch_bounds__(256, MINB) void k_conv_mfma(conv_args a)
{
    constexpr int KS = CIN / 16;             // MFMA k-steps per tap
    constexpr int NCH = CIN / 8;             // 16-byte channel groups per input pixel
    constexpr int PIXB = CIN * 2;            // bytes per input pixel
    constexpr int PH = TH + 2;
    constexpr int RW = TH / 4;               // rows per wave
    constexpr int NR = RW + 2;               // input rows per wave
    constexpr int WBYTES = 9 * KS * MT * 1024;
    constexpr int SWZ_SH = (NCH == 8) ? 0 : 1;
    constexpr int NSTEP = 3 * KS;
    constexpr int CQ = 32 * MT;              // channels of one output pixel (bf16 mode)
    // patch pieces (16 bytes each) of a thread: the 32 inner columns of patch row RPJ*j + m_row
    // are PPR contiguous pieces in global memory; the 2 halo columns are NHALO extra pieces
    constexpr int PPR = 32 * NCH, RPJ = 256 / PPR, NMAIN = PH / RPJ;
    constexpr int NHP = PH * 2 * NCH, NHALO = (NHP + 255) / 256, NPRE = NMAIN + NHALO;
    static_assert(PH % RPJ == 0, "patch rows must split evenly over the threads");
    // output pieces of a lane (bf16 mode): pixel (j*64 + lane) / NCHO of the wave's RW x 32 pixels
    constexpr int NCHO = CQ / 8, OPIXB = CQ * 2, OSH = (NCHO == 8) ? 0 : 1;
    constexpr int NOUT = F32OUT ? 0 : RW * 32 * NCHO / 64, PPJ = 64 / NCHO, JPR = 32 / PPJ;
    // issue schedule of the global memory instructions over the MFMA steps
    constexpr int ST_STEPS = NSTEP * 2 / 3, SK_STEPS = NSTEP - ST_STEPS, LD_STEPS = NSTEP * 5 / 6;
    constexpr int SPS = F32OUT ? 0 : (NOUT + ST_STEPS - 1) / ST_STEPS, KPS = F32OUT ? 0 : (NOUT + SK_STEPS - 1) / SK_STEPS;
    constexpr int LPS = (NPRE + LD_STEPS - 1) / LD_STEPS;

    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* lds_w = lds;
    uint8_t* lds_p = lds + WBYTES;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int lx = lane & 31, hi = lane >> 5;
    const int n_img = a.n_valid ? min((int)*a.n_valid, a.N) : a.N;
    const int tiles_x = (a.W + TW - 1) / TW, tiles_y = (a.H + TH - 1) / TH;
    const int tiles_img = tiles_x * tiles_y;
    const int n_tiles = n_img * tiles_img;
    // consecutive tiles go to workgroups of one XCD (workgroups are dealt round-robin to the 8 XCDs)
    const int G = gridDim.x;
    const int wg = (G % 8 == 0) ? (blockIdx.x % 8) * (G / 8) + blockIdx.x / 8 : blockIdx.x;
    const int ps = a.ps;
    const uint32_t in_img_bytes = (uint32_t)a.H * a.W * PIXB;
    const uint32_t out_img_bytes = F32OUT ? 0u : (uint32_t)(a.H * ps) * (a.W * ps) * OPIXB;

    // per-thread constants of the patch pieces
    const int m_row = tid / PPR, m_col = (tid % PPR) / NCH, m_c = tid % NCH;
    const int m_goff = (m_row * a.W + m_col) * PIXB + m_c * 16;                    // + tile origin + j rows
    const uint32_t m_lds = (uint32_t)(m_row * (PW * PIXB) + (1 + m_col) * PIXB + ((m_c ^ (((1 + m_col) >> SWZ_SH) & (NCH - 1))) << 4));
    // per-lane constants of the output pieces
    const int lcol = lane / (F32OUT ? 1 : NCHO), lc = lane % (F32OUT ? 1 : NCHO);
    const int o_lane = (lcol * ps) * OPIXB + lc * 16;
    const int o_rowpitch = a.W * ps * OPIXB;

    uint4 pre[NPRE];
    // patch piece j of tile (y0, x0) of the image behind rin
    auto load_piece = [&](int j, __amdgpu_buffer_rsrc_t rin, int y0, int x0) __attribute__((always_inline)) {
        int off; bool ok;
        if (j < NMAIN) {
            const int gy = y0 - 1 + RPJ * j + m_row;
            ok = gy >= 0 && gy < a.H && x0 + m_col < a.W;
            off = ((y0 - 1 + RPJ * j) * a.W + x0) * PIXB + m_goff;
        } else {
            const int idx = tid + 256 * (j - NMAIN), row = idx / (2 * NCH), side = (idx / NCH) & 1, c = idx % NCH;
            const int gy = y0 - 1 + row, hx = side ? x0 + TW : x0 - 1;
            ok = idx < NHP && gy >= 0 && gy < a.H && hx >= 0 && hx < a.W;
            off = (gy * a.W + hx) * PIXB + c * 16;
        }
        const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rin, ok ? (uint32_t)off : OOB_OFF, 0, 0);
        pre[j] = make_uint4(v[0], v[1], v[2], v[3]);
    };
    auto store_patch = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NMAIN; ++j) *(uint4*)(lds_p + j * (RPJ * PW * PIXB) + m_lds) = pre[j];
#pragma unroll
        for (int j = 0; j < NHALO; ++j) {
            const int idx = tid + 256 * j, row = idx / (2 * NCH), side = (idx / NCH) & 1, c = idx % NCH;
            const int px = side ? PW - 1 : 0;
            if (idx < NHP) *(uint4*)(lds_p + (row * PW + px) * PIXB + ((c ^ ((px >> SWZ_SH) & (NCH - 1))) << 4)) = pre[NMAIN + j];
        }
    };
    // byte offset of output piece j of tile (y0, x0) inside its image, or OOB_OFF outside the image
    auto out_off = [&](int j, int y0, int x0, int si, int sj) __attribute__((always_inline)) {
        const int y = y0 + wave * RW + j / JPR, xb = x0 + (j % JPR) * PPJ;
        const bool ok = y < a.H && xb + lcol < a.W;
        const int off = (y * ps + si) * o_rowpitch + (xb * ps + sj) * OPIXB + o_lane;
        return ok ? (uint32_t)off : OOB_OFF;
    };

    for (int chunk = 0; chunk < a.n_chunks; ++chunk) {
        __syncthreads();
        {   // this chunk's weights -> LDS
            const uint4* src = a.wp + (size_t)chunk * (WBYTES / 16);
            for (int i = tid; i < WBYTES / 16; i += 256) ((uint4*)lds_w)[i] = src[i];
        }
        // bias in accumulator layout: lane holds channels m*32 + 8*(e/4) + 4*hi + e%4
        f32x16 biasv[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int e = 0; e < 16; ++e) biasv[m][e] = a.bias[chunk * CQ + m * 32 + (e >> 2) * 8 + hi * 4 + (e & 3)];
        const int si = chunk / ps, sj = chunk - si * ps;

        int tile = wg;
        if (tile < n_tiles) {
            const int n = tile / tiles_img, tr = tile - n * tiles_img, ty = tr / tiles_x, tx = tr - ty * tiles_x;
            __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc((void*)(a.in + (size_t)n * a.H * a.W * CIN), 0, in_img_bytes, RSRC_FLAGS);
#pragma unroll
            for (int j = 0; j < NPRE; ++j) load_piece(j, rin, ty * TH, tx * TW);
        }
        uint4 outv[F32OUT ? 1 : NOUT];       // previous tile's result, stored during this tile's MFMA loop
        int out_tile = -1;
        for (; tile < n_tiles; tile += G) {
            const int n = tile / tiles_img, tr = tile - n * tiles_img;
            const int ty = tr / tiles_x, tx = tr - ty * tiles_x;
            const int y0 = ty * TH, x0 = tx * TW;
            lds_barrier();                                     // (A) LDS reads of the previous tile are done
            store_patch();
            lds_barrier();                                     // (B)
            // descriptors: next tile's input image (empty if there is no next tile), previous
            // tile's output image (empty if none), this tile's skip image
            const int nt = tile + G;
            const bool has_next = nt < n_tiles;
            const int nn = has_next ? nt / tiles_img : 0, ntr = nt - nn * tiles_img, nty = ntr / tiles_x, ntx = ntr - nty * tiles_x;
            __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc(
                (void*)(a.in + (size_t)nn * a.H * a.W * CIN), 0, has_next ? in_img_bytes : 0u, RSRC_FLAGS);
            const int on = out_tile >= 0 ? out_tile / tiles_img : 0, otr = out_tile - on * tiles_img, oty = otr / tiles_x, otx = otr - oty * tiles_x;
            __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc(
                (void*)((uint8_t*)a.out + (size_t)on * out_img_bytes), 0, out_tile >= 0 ? out_img_bytes : 0u, RSRC_FLAGS);
            __amdgpu_buffer_rsrc_t rsk = __builtin_amdgcn_make_buffer_rsrc(
                (void*)((uint8_t*)a.skip + (size_t)n * out_img_bytes), 0, SKIP ? out_img_bytes : 0u, RSRC_FLAGS);
            uint4 sk[(SKIP && !F32OUT) ? NOUT : 1];

            f32x16 acc[RW][MT];
            const uint8_t* wlane = lds_w + (lane << 4);
            const uint8_t* prow = lds_p + (wave * RW) * (PW * PIXB);
            auto load_A = [&](int st, bf16x8 (&A)[3][MT]) __attribute__((always_inline)) {
                const int kx = st / KS, ks = st - kx * KS;
#pragma unroll
                for (int ky = 0; ky < 3; ++ky)
#pragma unroll
                    for (int m = 0; m < MT; ++m)
                        A[ky][m] = *(const bf16x8*)(wlane + ((((ky * 3 + kx) * KS + ks) * MT + m) << 10));
            };
            auto load_B = [&](int st, bf16x8 (&B)[NR]) __attribute__((always_inline)) {
                const int kx = st / KS, ks = st - kx * KS;
                const int px = lx + kx;
                const int key = (px >> SWZ_SH) & (NCH - 1);
                const uint8_t* b0 = prow + px * PIXB + (((2 * ks + hi) ^ key) << 4);
#pragma unroll
                for (int py = 0; py < NR; ++py) B[py] = *(const bf16x8*)(b0 + py * (PW * PIXB));
            };
            bf16x8 A0[3][MT], A1[3][MT], B0[NR], B1[NR];
            load_A(0, A0); load_B(0, B0);
            // One step, cut into NSLOT slots.  Every slot issues its share of the next step's
            // fragment loads and at most one global memory instruction, then its MFMAs; the
            // scheduling barrier after a slot keeps that interleaving in the instruction stream.
            auto step = [&](auto st_c) __attribute__((always_inline)) {
                constexpr int st = decltype(st_c)::value;
                constexpr int NMF = 3 * RW * MT, NFR = 3 * MT + NR, NSLOT = 6;
                constexpr int MPS = NMF / NSLOT, FPS = (NFR + NSLOT - 1) / NSLOT;
                static_assert(NMF % NSLOT == 0, "MFMAs of a step must split evenly over the slots");
                bf16x8 (&Ac)[3][MT] = (st & 1) ? A1 : A0;
                bf16x8 (&Bc)[NR] = (st & 1) ? B1 : B0;
                bf16x8 (&An)[3][MT] = (st & 1) ? A0 : A1;
                bf16x8 (&Bn)[NR] = (st & 1) ? B0 : B1;
                constexpr int kxn = (st + 1) / KS, ksn = (st + 1) - kxn * KS;
                const int pxn = lx + kxn;
                const uint8_t* b0n = prow + pxn * PIXB + (((2 * ksn + hi) ^ ((pxn >> SWZ_SH) & (NCH - 1))) << 4);
                constexpr int n_st = (!F32OUT && st < ST_STEPS) ? SPS : 0;          // stores in this step
                constexpr int n_ld = (st < LD_STEPS) ? LPS : 0;                     // patch loads
                constexpr int n_sk = (SKIP && !F32OUT && st >= ST_STEPS) ? KPS : 0; // skip loads
                static_assert(n_st + n_ld + n_sk <= NSLOT, "too many memory instructions for one step");
#pragma unroll
                for (int sl = 0; sl < NSLOT; ++sl) {
                    if (st + 1 < NSTEP) {
#pragma unroll
                        for (int f = sl * FPS; f < (sl + 1) * FPS && f < NFR; ++f) {
                            if (f < 3 * MT) An[f / MT][f % MT] = *(const bf16x8*)(wlane + (((((f / MT) * 3 + kxn) * KS + ksn) * MT + f % MT) << 10));
                            else Bn[f - 3 * MT] = *(const bf16x8*)(b0n + (f - 3 * MT) * (PW * PIXB));
                        }
                    }
                    if (sl < n_st) {
                        const int j = st * SPS + sl;
                        if (j < NOUT) {
                            const i32x4 v = {(int)outv[j].x, (int)outv[j].y, (int)outv[j].z, (int)outv[j].w};
                            __builtin_amdgcn_raw_buffer_store_b128(v, rout, out_off(j, oty * TH, otx * TW, si, sj), 0, 0);
                        }
                    } else if (sl < n_st + n_ld) {
                        const int j = st * LPS + (sl - n_st);
                        if (j < NPRE) load_piece(j, rin, nty * TH, ntx * TW);
                    } else if (sl < n_st + n_ld + n_sk) {
                        const int j = (st - ST_STEPS) * KPS + (sl - n_st - n_ld);
                        if (j < NOUT) {
                            const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rsk, out_off(j, y0, x0, 0, 0), 0, 0);
                            sk[j] = make_uint4(v[0], v[1], v[2], v[3]);
                        }
                    }
#pragma unroll
                    for (int k = sl * MPS; k < (sl + 1) * MPS; ++k) {
                        // MFMA k of the step: (input row py, tap ky) pairs with 0 <= py - ky < RW, py-major
                        const int m = k % MT, pair = k / MT;
                        int py = 0, ky = 0, cnt = 0;
#pragma unroll
                        for (int p = 0; p < NR; ++p)
#pragma unroll
                            for (int q = 0; q < 3; ++q)
                                if (p - q >= 0 && p - q < RW) { if (cnt == pair) { py = p; ky = q; } ++cnt; }
                        const int r = py - ky;
                        acc[r][m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ac[ky][m], Bc[py], (st == 0 && ky == 0) ? biasv[m] : acc[r][m], 0, 0, 0);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                }
            };
            for_each_step<NSTEP>(step);
            // lane holds, for pixel column lx of each of its rows, channels
            // m*32 + 8*q + 4*hi + {0,1,2,3} in acc[r][m][4q..4q+3]
            if constexpr (F32OUT) {
                const int x = x0 + lx;
                const int s = a.s_final, s2 = s * s;
                float* o = (float*)a.out;
#pragma unroll
                for (int r = 0; r < RW; ++r) {
                    const int y = y0 + wave * RW + r;
                    if (y >= a.H || x >= a.W) continue;
#pragma unroll
                    for (int m = 0; m < MT; ++m)
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const int cb = m * 32 + q * 8 + hi * 4;
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                const int co = cb + e;
                                if (co >= a.cout_real) continue;
                                const int ch = co / s2, sub = co - ch * s2, ui = sub / s, uj = sub - ui * s;
                                o[(((size_t)n * a.H * s + (size_t)y * s + ui) * (a.W * s) + (size_t)x * s + uj) * 3 + ch] = acc[r][m][4 * q + e];
                            }
                        }
                }
            } else {
                lds_barrier();                             // (C) every wave is done with the patch
                uint8_t* stg = lds_p + wave * (RW * 32 * OPIXB);
                const int okey = (lx >> OSH) & (NCHO - 1);
#pragma unroll
                for (int m = 0; m < MT; ++m)
#pragma unroll
                    for (int q = 0; q < 4; ++q)
#pragma unroll
                        for (int r = 0; r < RW; ++r) {
                            float v0 = acc[r][m][4 * q + 0], v1 = acc[r][m][4 * q + 1], v2 = acc[r][m][4 * q + 2], v3 = acc[r][m][4 * q + 3];
                            uint2 pk;
                            pk.x = pack_bf16x2(v0, v1); pk.y = pack_bf16x2(v2, v3);
                            if constexpr (RELU) { pk.x = relu_bf16x2(pk.x); pk.y = relu_bf16x2(pk.y); }
                            *(uint2*)(stg + (r * 32 + lx) * OPIXB + (((m * 4 + q) ^ okey) << 4) + hi * 8) = pk;
                        }
                lds_barrier();                             // (D) staged values visible
#pragma unroll
                for (int j = 0; j < NOUT; ++j) {
                    const int r = j / JPR, px = (j % JPR) * PPJ + lcol;
                    uint4 o = *(const uint4*)(stg + (r * 32 + px) * OPIXB + ((lc ^ ((px >> OSH) & (NCHO - 1))) << 4));
                    if constexpr (SKIP) {
                        o.x = pack_bf16x2(bf16_lo(o.x) + bf16_lo(sk[j].x), bf16_hi(o.x) + bf16_hi(sk[j].x));
                        o.y = pack_bf16x2(bf16_lo(o.y) + bf16_lo(sk[j].y), bf16_hi(o.y) + bf16_hi(sk[j].y));
                        o.z = pack_bf16x2(bf16_lo(o.z) + bf16_lo(sk[j].z), bf16_hi(o.z) + bf16_hi(sk[j].z));
                        o.w = pack_bf16x2(bf16_lo(o.w) + bf16_lo(sk[j].w), bf16_hi(o.w) + bf16_hi(sk[j].w));
                    }
                    outv[j] = o;
                }
                out_tile = tile;
            }
        }
        if constexpr (!F32OUT) {
            if (out_tile >= 0) {                           // the last tile's result
                const int on = out_tile / tiles_img, otr = out_tile - on * tiles_img, oty = otr / tiles_x, otx = otr - oty * tiles_x;
                __amdgpu_buffer_rsrc_t rout = __builtin_amdgcn_make_buffer_rsrc((void*)((uint8_t*)a.out + (size_t)on * out_img_bytes), 0, out_img_bytes, RSRC_FLAGS);
#pragma unroll
                for (int j = 0; j < NOUT; ++j) {
                    const i32x4 v = {(int)outv[j].x, (int)outv[j].y, (int)outv[j].z, (int)outv[j].w};
                    __builtin_amdgcn_raw_buffer_store_b128(v, rout, out_off(j, oty * TH, otx * TW, si, sj), 0, 0);
                }
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// host side

static uint16_t f32_to_bf16_rne(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

// Repack every layer with cin = C into fragment order:
//   [chunk][tap][ks][m][lane][8]  with  cout' = chunk*CQ + m*32 + lane%32,
//   ci = ks*16 + 8*(lane/32) + e,   cout' -> original cout through the pixel-shuffle fold.
rh_status rh_pack_weights_bf16(rh_ctx* ctx, const float* blob)
{
    const int C = ctx->cfg.net.channels, s = ctx->cfg.net.scale;
    if (C != 32 && C != 64) RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "bf16 path supports 32 or 64 channels, got %d", C);
    std::vector<uint16_t> wp;
    std::vector<float> bp;
    const size_t nl = ctx->layers.size();
    for (size_t li = 0; li < nl; ++li) {
        rh_layer& L = ctx->layers[li];
        L.wp_off = wp.size() * 2; L.bp_off = bp.size();
        const float* w = blob + L.w_off; const float* b = blob + L.b_off;
        if (L.cin == 3) {                      // head: [ky][m][lane][8], row = cout, k = 8*(lane/32) + e = kx*3 + c (>= 9: zero)
            L.cout_pad = L.cout; L.ps = 1;
            for (int ky = 0; ky < 3; ++ky)
                for (int m = 0; m < L.cout / 32; ++m)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int e = 0; e < 8; ++e) {
                            const int co = m * 32 + (lane & 31), j = 8 * (lane >> 5) + e;
                            wp.push_back(f32_to_bf16_rne(j < 9 ? w[((size_t)co * 3 + ky) * 9 + j] : 0.0f));
                        }
            for (int co = 0; co < L.cout; ++co) bp.push_back(b[co]);
            continue;
        }
        const bool last = (li == nl - 1);
        L.tail3 = 0;
        if (last && L.cout == 3) {             // [ks][lane][8]: row m = lane%32 = tap*3 + co, ci = 16*ks + 8*(lane/32) + e
            L.tail3 = 1; L.cout_pad = 32; L.ps = 1;
            for (int ks = 0; ks < L.cin / 16; ++ks)
                for (int lane = 0; lane < 64; ++lane)
                    for (int e = 0; e < 8; ++e) {
                        const int m = lane & 31, tap = m / 3, co = m - tap * 3;
                        const int ci = ks * 16 + 8 * (lane >> 5) + e;
                        wp.push_back(f32_to_bf16_rne(m < 27 ? w[((size_t)co * 9 + tap) * L.cin + ci] : 0.0f));
                    }
            for (int co = 0; co < 4; ++co) bp.push_back(co < 3 ? b[co] : 0.0f);
            continue;
        }
        int ps = 1;
        if (!last && L.cout != C) {            // upsampling conv: cout = C * r^2
            ps = (L.cout == 4 * C) ? 2 : (L.cout == 9 * C ? 3 : 0);
            if (!ps) RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "unexpected layer shape %d->%d", L.cin, L.cout);
        }
        L.ps = ps;
        const int CQ = last ? ((L.cout + 31) / 32) * 32 : C;     // channels per chunk
        if (CQ > 64) RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "last conv with %d outputs (scale %d) exceeds 64", L.cout, s);
        const int n_chunks = last ? 1 : ps * ps, MT = CQ / 32, KS = L.cin / 16;
        L.cout_pad = CQ * n_chunks;
        for (int q = 0; q < n_chunks; ++q)
            for (int tap = 0; tap < 9; ++tap)
                for (int ks = 0; ks < KS; ++ks)
                    for (int m = 0; m < MT; ++m)
                        for (int lane = 0; lane < 64; ++lane)
                            for (int e = 0; e < 8; ++e) {
                                const int cp = m * 32 + (lane & 31);             // channel within the chunk
                                const int co = last ? cp : (ps == 1 ? cp : cp * ps * ps + q);
                                const int ci = ks * 16 + 8 * (lane >> 5) + e;
                                float v = (co < L.cout) ? w[((size_t)co * 9 + tap) * L.cin + ci] : 0.0f;
                                wp.push_back(f32_to_bf16_rne(v));
                            }
        for (int q = 0; q < n_chunks; ++q)
            for (int cp = 0; cp < CQ; ++cp) {
                const int co = last ? cp : (ps == 1 ? cp : cp * ps * ps + q);
                bp.push_back(co < L.cout ? b[co] : 0.0f);
            }
    }
    RH_HIP(ctx, hipMalloc(&ctx->wpack, wp.size() * 2 + 16));
    RH_HIP(ctx, hipMalloc((void**)&ctx->bpack, bp.size() * 4 + 16));
    RH_HIP(ctx, hipMemcpy(ctx->wpack, wp.data(), wp.size() * 2, hipMemcpyHostToDevice));
    RH_HIP(ctx, hipMemcpy(ctx->bpack, bp.data(), bp.size() * 4, hipMemcpyHostToDevice));
    return RH_OK;
}

template <int CIN, int MT, int TH, bool F32OUT, bool SKIP, bool RELU, int MINB = 1>
static hipError_t launch_conv(rh_ctx* ctx, const conv_args& a, int grid)
{
    constexpr int lds = 9 * (CIN / 16) * MT * 1024 + (TH + 2) * PW * CIN * 2;
    static bool attr_done[RH_MAX_DEVICES] = {};            // the attribute is per device
    if (!attr_done[ctx->device]) {
        hipError_t e = hipFuncSetAttribute((const void*)k_conv_mfma<CIN, MT, TH, F32OUT, SKIP, RELU, MINB>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_done[ctx->device] = true;
    }
    hipLaunchKernelGGL((k_conv_mfma<CIN, MT, TH, F32OUT, SKIP, RELU, MINB>), dim3(grid), dim3(256), lds, ctx->stream, a);
    return hipSuccess;
}

static rh_status conv(rh_ctx* ctx, const rh_layer& L, const __bf16* in, void* out, const __bf16* skip, int N, int H,
                      int W, int relu, bool last, int s_final, const uint32_t* n_valid)
{
    conv_args a;
    a.in = in; a.wp = (const uint4*)((const uint8_t*)ctx->wpack + L.wp_off); a.bias = ctx->bpack + L.bp_off;
    a.out = out; a.skip = skip; a.n_valid = n_valid; a.N = N; a.H = H; a.W = W;
    a.relu = relu; a.ps = L.ps; a.n_chunks = last ? 1 : L.ps * L.ps; a.cout_real = L.cout; a.s_final = s_final;
    a.rev = (ctx->conv_parity ^= 1);       // alternate the direction from one conv to the next
    // box-masked mode: the body's convs (same resolution in and out) walk the live cells only
    const bool body = !last && L.ps == 1 && L.cin == 64;
    a.tile_list = nullptr; a.n_list = nullptr;
    if (ctx->mk_boxes && body) { a.tile_list = ctx->cell_live; a.n_list = ctx->cell_cnt; }
    // needed-region mode: the cells within this conv's radius of a placed macroblock
    if (ctx->nd_places && body) {
        const int r = ctx->nd_radii[1 + ctx->nd_conv++];
        if (r <= RH_NEED_RMAX) { a.tile_list = ctx->need_lists + (size_t)r * ctx->need_cap; a.n_list = ctx->need_cnt + r; }
    }
    const int grid = ctx->n_cu;            // persistent kernels: one workgroup per compute unit (256 on MI355X)
    const int MT = last ? L.cout_pad / 32 : L.cin / 32;
    hipError_t e;
    // bf16-output convs come as (ReLU, no skip), (skip, no ReLU) or (neither)
    if (last && L.tail3 && s_final == 1) e = rh_launch_conv_tail3(ctx->stream, ctx->device, a, L.cin);
    else if (last && L.tail3) RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "3-channel last conv with a pixel shuffle");
    else if (L.cin == 64) {
        if (last) e = (MT == 2) ? launch_conv<64, 2, 16, true, false, false>(ctx, a, grid) : launch_conv<64, 1, 8, true, false, false, 2>(ctx, a, 2 * grid);
        else e = rh_launch_conv_duo(ctx->stream, ctx->device, a, grid, skip != nullptr, relu != 0);    // two-team kernel
    } else {
        if (last) e = (MT == 2) ? launch_conv<32, 2, 16, true, false, false>(ctx, a, grid) : launch_conv<32, 1, 16, true, false, false>(ctx, a, grid);
        else if (skip) e = launch_conv<32, 1, 16, false, true, false>(ctx, a, grid);
        else if (relu) e = launch_conv<32, 1, 16, false, false, true>(ctx, a, grid);
        else e = launch_conv<32, 1, 16, false, false, false>(ctx, a, grid);
    }
    RH_HIP(ctx, e);
    return RH_OK;
}

rh_status rh_launch_enhance_bf16(rh_ctx* ctx, const uint8_t* in, int N, int H, int W, float* out,
                                 const uint32_t* n_valid)
{
    const rh_net_desc& d = ctx->cfg.net;
    const int C = d.channels, s = d.scale;
    const size_t lr = (size_t)N * H * W * C;
    size_t need = 3 * lr, up1 = 0, up2 = 0;
    // the composed upsampler + last conv replaces the per-layer run, except in exact-border mode
    // (which clears the out-of-frame activations of every layer it would skip)
    const bool fold = d.topology == RH_NET_EDSR && ctx->fold_chunks > 0 && !ctx->bz_boxes;
    if (d.topology == RH_NET_EDSR && !fold) {
        const int r = (s == 4) ? 2 : s;
        up1 = lr * r * r; need += up1;
        if (s == 4) { up2 = up1 * 4; need += up2; }
    }
    {   // the conv kernels address one image with 32-bit byte offsets (buffer instructions)
        const int rmax = (d.topology == RH_NET_EDSR && !fold) ? s : 1;
        const unsigned long long img_bytes = (unsigned long long)H * rmax * W * rmax * C * 2ull;
        if (img_bytes >= (1ull << 31))
            RH_FAIL(ctx, RH_E_SHAPE, "rh_enhance: %dx%d images need %llu bytes of bf16 activations each at x%d; the limit is 2 GiB",
                    W, H, img_bytes, rmax);
    }
    rh_status st = rh_ensure_workspace(ctx, need * 2);
    if (st != RH_OK) return st;
    __bf16* a = (__bf16*)ctx->act; __bf16* t = a + lr; __bf16* h = t + lr; __bf16* u1 = h + lr; __bf16* u2 = u1 + up1;
    ctx->conv_parity = 0;                  // the head conv walks forward, the first conv after it backward
    const std::vector<rh_layer>& L = ctx->layers;
    size_t li = 0;
    const int head_relu = d.topology == RH_NET_PLAIN;
    {
        const rh_layer& l0 = L[li++];
        rh_prof_scope ps(ctx, RH_PROF_HEAD);
        RH_HIP(ctx, rh_launch_head_mfma(ctx->stream, C, in, (const uint4*)((const uint8_t*)ctx->wpack + l0.wp_off),
                                        ctx->bpack + l0.bp_off, h, N, H, W, head_relu, n_valid));
        // box-masked mode: from here to the end of the body the three tensors are zero outside the live cells
        if (ctx->mk_boxes) { st = rh_launch_cell_lists(ctx, N, n_valid, h, a, t); if (st != RH_OK) return st; }
        if (ctx->nd_places) { ctx->nd_conv = 0; st = rh_launch_need_lists(ctx, N, n_valid); if (st != RH_OK) return st; }
    }
    // exact-border mode (a no-op otherwise): clear the out-of-frame part of the boxes in a layer's output
#define ZERO(buf, res) do { st = rh_zero_outside(ctx, (void*)(buf), C * 2, (res), N, n_valid); if (st != RH_OK) return st; } while (0)
    ZERO(h, 1);
    // one event pair around the run of bf16-output convs (they are launched back to back) and
    // one around the last conv: per-launch events would put a bubble between the launches
    uint32_t n_conv = 0;
    rh_prof_begin(ctx, RH_PROF_CONV);
#define CONV(...) do { st = conv(ctx, __VA_ARGS__); if (st != RH_OK) return st; ++n_conv; } while (0)
#define LAST_CONV(...) do { rh_prof_end(ctx, n_conv); rh_prof_scope ps_(ctx, RH_PROF_CONV_LAST); st = conv(ctx, __VA_ARGS__); if (st != RH_OK) return st; } while (0)
    if (d.topology == RH_NET_PLAIN) {
        const __bf16* x = h;
        for (int l = 0; l < d.n_blocks - 2; ++l) { __bf16* o = (x == a) ? t : a; CONV(L[li++], x, o, nullptr, N, H, W, 1, false, 1, n_valid); ZERO(o, 1); x = o; }
        LAST_CONV(L[li++], x, out, nullptr, N, H, W, 0, true, s, n_valid);
    } else {
        const __bf16* x = h;
        for (int b = 0; b < d.n_blocks; ++b) {
            CONV(L[li++], x, t, nullptr, N, H, W, 1, false, 1, n_valid); ZERO(t, 1);
            CONV(L[li++], t, a, x, N, H, W, 0, false, 1, n_valid); ZERO(a, 1);      // x + conv(t)
            x = a;
        }
        if (d.topology == RH_NET_RES) {
            LAST_CONV(L[li++], x, out, nullptr, N, H, W, 0, true, s, n_valid);
        } else {
            CONV(L[li++], x, t, h, N, H, W, 0, false, 1, n_valid); ZERO(t, 1);       // body end + long skip
            if (fold) {
                rh_prof_end(ctx, n_conv);
                rh_prof_scope ps_(ctx, RH_PROF_CONV_LAST, 2);
                // needed-region mode: the composed tail's output is needed on the pasted macroblocks only (radius 0)
                st = rh_launch_fold(ctx, t, out, N, H, W, n_valid, ctx->conv_parity ^= 1,
                                    ctx->nd_places ? ctx->need_lists : nullptr, ctx->nd_places ? ctx->need_cnt : nullptr);
                if (st != RH_OK) return st;
            } else {
                const int r = (s == 4) ? 2 : s;
                CONV(L[li++], t, u1, nullptr, N, H, W, 0, false, 1, n_valid); ZERO(u1, r);
                const __bf16* lastin = u1; int hh = H * r, ww = W * r;
                if (s == 4) { CONV(L[li++], u1, u2, nullptr, N, hh, ww, 0, false, 1, n_valid); ZERO(u2, 2 * r); lastin = u2; hh *= 2; ww *= 2; }
                LAST_CONV(L[li++], lastin, out, nullptr, N, hh, ww, 0, true, 1, n_valid);
            }
        }
    }
#undef CONV
#undef LAST_CONV
#undef ZERO
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

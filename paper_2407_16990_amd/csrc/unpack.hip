// Paste (Sec. 3.3.3) fused with the bilinear base IN(.) of the problem statement
// (Sec. 3.2.1): one pass writes every high-resolution pixel exactly once.  For a placed
// macroblock the pixel is clamp(base/255 + net) quantised, otherwise the base itself.
#include "rh_internal.h"

__global__ __launch_bounds__(256) void k_identity_places(rh_mbplace* __restrict__ places, uint32_t* __restrict__ n_places,
                                                         int mbw, int per, uint32_t total)
{
    const uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g == 0) *n_places = total;
    if (g >= total) return;
    const uint32_t f = g / per, in = g % per;
    rh_mbplace p;
    p.mb_id = g; p.box = f; p.bin = (uint16_t)f; p.px = (uint16_t)(RH_MB * (in % mbw)); p.py = (uint16_t)(RH_MB * (in / mbw)); p.rot = 0;
    places[g] = p;
}

// Bilinear base + paste for integer scale S, one launch.  A workgroup writes a strip of NMBX
// macroblocks (one macroblock row tall): the 64 lanes of a wave lie side by side along x, 4 output
// pixels (12 bytes) each, so a wave instruction writes up to 768 contiguous bytes; the 4 waves
// split the 16 input rows.
// Input tile (18 rows, clamped at the frame edge): fetched as aligned 4-byte words, every thread
// issuing all of its loads before it waits for one; a row's words land in LDS as they are and the
// row's byte shift (frame rows start at arbitrary byte addresses) is applied when pixels are read.
// Placement lookup: `places` is ascending in mb_id, so the rows of the strip's macroblocks are
// found by a 64-ary search in which the lanes of a wave probe 64 rows at a time (two or three
// dependent loads for any batch size); no per-call index table is built.
// Exact integer interpolation: weights are multiples of 1/(2S) in each direction,
// out = (sum + D*D/2) / (D*D) with D = 2S; all intermediate values fit 16 bits (255 * D * D +
// D*D/2 <= 16352), so the arithmetic runs on packed pairs.  For a placed macroblock the pixel
// becomes floor(255 * clamp(base/255 + net, 0, 1) + 0.5) in fp32 (base/255 from a 256-entry table
// of correctly rounded quotients).
// EDGE: frames with cut macroblocks at the right / bottom edge (sides not multiples of 16) or a row
// pitch that is not a multiple of 4 bytes; those blocks go pixel by pixel.  A place is honoured
// when the in-frame part of its block lies inside the enhanced image (for whole macroblocks:
// px + 16 <= iw and py + 16 <= ih), otherwise the macroblock stays bilinear.
typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

template <int S, bool EDGE>
__global__ __launch_bounds__(256) void k_unpack(const uint8_t* __restrict__ lr, int H, int W, int mbw,
                                                const float* __restrict__ enh, int n_img, int ih, int iw,
                                                const rh_mbplace* __restrict__ places,
                                                const uint32_t* __restrict__ n_places, uint32_t cap,
                                                uint8_t* __restrict__ hr, float* __restrict__ sel)
{
    constexpr int B = RH_MB * S, D = 2 * S, GPM = B / 4, NMBX = 64 / GPM, LANES = NMBX * GPM;
    constexpr int TWID = RH_MB * NMBX + 2;                   // tile width in pixels
    constexpr int TPD = (TWID * 3 + 3 + 3) / 4 + 1;          // 4-byte words per tile row, any byte shift
    constexpr int NLD = (18 * TPD + 255) / 256;              // words per thread
    __shared__ uint32_t tile[18][TPD];
    __shared__ float q255[256];
    const int strip = blockIdx.x, my = blockIdx.y, f = blockIdx.z, tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6, mbh = gridDim.y;
    const int lx0 = RH_MB * NMBX * strip - 1;                // frame column of tile pixel 0 (may be -1)
    const int xs = max(lx0, 0), xe = min(lx0 + TWID, W);     // columns [xs, xe) are fetched
    // ---- issue the tile's loads ----
    uint32_t tw[NLD];
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int idx = j * 256 + tid, row = idx / TPD, d = idx - row * TPD;
        tw[j] = 0;
        if (row < 18) {
            const int y = min(max(RH_MB * my - 1 + row, 0), H - 1);
            const uintptr_t beg = (uintptr_t)lr + (((size_t)f * H + y) * W + xs) * 3, end = beg + (size_t)(xe - xs) * 3;
            const uintptr_t wa = (beg & ~(uintptr_t)3) + 4u * (uintptr_t)d;      // holds at least one byte of the row
            if (wa < end) tw[j] = *(const uint32_t*)wa;
        }
    }
    // ---- placement rows of the strip's macroblocks: 64-ary lower bound of the first one ----
    const uint32_t g0 = ((uint32_t)f * mbh + my) * mbw + strip * NMBX;
    const uint32_t n = min(*n_places, cap);
    uint32_t lo = 0, hi = n;                                 // rows < lo have mb_id < g0, rows >= hi have mb_id >= g0
    while (hi - lo > 64u - NMBX) {                           // uniform over the wave
        const uint32_t step = (hi - lo + 63u) / 64u, p = lo + (uint32_t)lane * step;
        const bool below = p < hi && places[p].mb_id < g0;
        const uint32_t cnt = (uint32_t)__popcll(__ballot(below));           // lanes 0 .. cnt-1 (the rows are ascending)
        const uint32_t nhi = lo + cnt * step;
        if (cnt < 64u && nhi < hi) hi = nhi;
        if (cnt) lo = lo + (cnt - 1u) * step + 1u;
    }
    // the lower bound lies in [lo, hi], hi - lo <= 64 - NMBX: rows lo .. lo+63 hold every macroblock of the strip
    uint4 row4 = make_uint4(0xFFFFFFFFu, 0, 0, 0);
    if (lo + (uint32_t)lane < n) row4 = *(const uint4*)(places + lo + lane);
    const int mbi = lane / GPM, mx = strip * NMBX + mbi;
    int slot = -1;
    uint32_t pl_bin_px = 0, pl_py_rot = 0;
#pragma unroll
    for (int j = 0; j < NMBX; ++j) {
        const unsigned long long m = __ballot(row4.x == g0 + (uint32_t)j);
        const int src = m ? __ffsll((long long)m) - 1 : 0;
        const uint32_t a2 = (uint32_t)__shfl((int)row4.z, src), a3 = (uint32_t)__shfl((int)row4.w, src);
        if (m && j == mbi) { slot = (int)lo + src; pl_bin_px = a2; pl_py_rot = a3; }
    }
    // ---- tile -> LDS ----
#pragma unroll
    for (int j = 0; j < NLD; ++j) {
        const int idx = j * 256 + tid;
        if (idx < 18 * TPD) (&tile[0][0])[idx] = tw[j];
    }
    q255[tid] = __fdiv_rn((float)tid, 255.0f);
    __syncthreads();
    if (lane >= LANES || mx >= mbw) return;
    const int gx = (lane - mbi * GPM) * 4;                // first of this lane's 4 pixels inside the macroblock
    const float* net = nullptr;
    bool turned = false;
    const int HW = W * S;
    const int fh = EDGE ? min(B, H * S - my * B) : B, fw = EDGE ? min(B, HW - mx * B) : B;   // in-frame part of the block
    if (slot >= 0) {
        const int p_bin = (int)(pl_bin_px & 0xFFFFu), p_px = (int)(pl_bin_px >> 16), p_py = (int)(pl_py_rot & 0xFFFFu);
        turned = (pl_py_rot >> 16) != 0;
        const int need_w = turned ? fh : fw, need_h = turned ? fw : fh;     // extent of that part inside the bin image
        if (p_bin != (int)RH_NO_BIN && p_bin < n_img && p_px * S + need_w <= iw * S && p_py * S + need_h <= ih * S) {
            // upright: this lane's first pixel of row 0; turned: the block's first pixel (rows and
            // columns are exchanged when reading)
            net = enh + (((size_t)p_bin * (ih * S) + (size_t)p_py * S) * (iw * S) + (size_t)p_px * S + (turned ? 0 : gx)) * 3;
        }
    }
    // horizontal taps of the 4 pixels: byte offset of the left neighbour inside a tile row (before
    // the row's shift), of the right one, and the right one's weight; columns clamp at the frame edge
    int o0[4], o1[4], wx1[4];
    const int row_sh0 = (int)(((uintptr_t)lr + ((size_t)f * H * W + xs) * 3) & 3u);     // shift of a row with y*W*3 = 0 (mod 4)
    const int pitch_sh = (W * 3) & 3;
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int nx = 2 * (gx + p) + 1 - S + D;          // shifted by one input pixel, always >= 0
        const int c0 = lx0 + nx / D + RH_MB * mbi;        // frame column of the left neighbour (-1 .. W-1)
        o0[p] = (min(max(c0, 0), W - 1) - xs) * 3; o1[p] = (min(c0 + 1, W - 1) - xs) * 3; wx1[p] = nx % D;
    }
    // horizontal sums of one tile row for the 4 pixels x 3 channels, as 6 packed pairs (k, k+6)
    auto hsum = [&](int row, u16x2 (&h)[6]) __attribute__((always_inline)) {
        const int y = min(max(RH_MB * my - 1 + row, 0), H - 1);
        const uint8_t* t = (const uint8_t*)&tile[row][0] + ((row_sh0 + y * pitch_sh) & 3);
        unsigned short v[12];
#pragma unroll
        for (int p = 0; p < 4; ++p)
#pragma unroll
            for (int c = 0; c < 3; ++c)
                v[p * 3 + c] = (unsigned short)((D - wx1[p]) * t[o0[p] + c] + wx1[p] * t[o1[p] + c]);
#pragma unroll
        for (int k = 0; k < 6; ++k) { h[k].x = v[k]; h[k].y = v[k + 6]; }
    };
    const bool edge = EDGE && (fh < B || fw < B || ((HW * 3) & 3));
    uint8_t* dst = hr + (((size_t)f * H * S + (size_t)my * B) * HW + (size_t)mx * B + gx) * 3;
    u16x2 h0[6], h1[6], h2[6];                             // input rows r-1, r, r+1 (tile rows r, r+1, r+2)
    const int r0 = wave * 4;
    hsum(r0, h0); hsum(r0 + 1, h1);
#pragma unroll
    for (int rr = 0; rr < 4; ++rr) {
        const int r = r0 + rr;
        hsum(r + 2, h2);
#pragma unroll
        for (int j = 0; j < S; ++j) {
            const int ny = 2 * j + 1 - S;                  // relative to input row r, in units of 1/D
            const int wy1 = ny < 0 ? ny + D : ny;
            const int yy = r * S + j;
            uint32_t bytes[12];
            const u16x2 wa = {(unsigned short)(D - wy1), (unsigned short)(D - wy1)}, wb = {(unsigned short)wy1, (unsigned short)wy1};
            const u16x2 rnd = {(unsigned short)(D * D / 2), (unsigned short)(D * D / 2)};
#pragma unroll
            for (int k = 0; k < 6; ++k) {
                const u16x2 acc = (ny < 0 ? h0[k] * wa + h1[k] * wb : h1[k] * wa + h2[k] * wb) + rnd;
                if constexpr ((D * D & (D * D - 1)) == 0) {
                    const u16x2 q = acc >> (unsigned short)__builtin_ctz(D * D);
                    bytes[k] = q.x; bytes[k + 6] = q.y;
                } else {
                    bytes[k] = (uint32_t)acc.x / (uint32_t)(D * D); bytes[k + 6] = (uint32_t)acc.y / (uint32_t)(D * D);
                }
            }
            if (EDGE && edge) {
                // Macroblock cut by the frame edge, or a row pitch that is not a multiple of 4 bytes:
                // pixel by pixel, bytes only where the frame is.
#pragma unroll
                for (int p = 0; p < 4; ++p) {
                    const int col = gx + p;
                    const bool in_frame = yy < fh && col < fw, pasted = net && in_frame;
                    float ev[3] = {0.0f, 0.0f, 0.0f};
                    if (pasted) {
                        const float* t = turned ? net + ((size_t)col * (iw * S) + yy) * 3 : net + ((size_t)yy * (iw * S) + p) * 3;
#pragma unroll
                        for (int c = 0; c < 3; ++c) {
                            ev[c] = fminf(fmaxf(__fadd_rn(q255[bytes[3 * p + c]], t[c]), 0.0f), 1.0f);
                            bytes[3 * p + c] = (uint32_t)__fadd_rn(__fmul_rn(ev[c], 255.0f), 0.5f);
                        }
                    }
                    if (net && sel) {
                        float* sp = sel + (((size_t)slot * B + yy) * B + col) * 3;
                        sp[0] = ev[0]; sp[1] = ev[1]; sp[2] = ev[2];
                    }
                    if (in_frame) {
                        uint8_t* o = dst + (size_t)yy * HW * 3 + p * 3;
                        o[0] = (uint8_t)bytes[3 * p]; o[1] = (uint8_t)bytes[3 * p + 1]; o[2] = (uint8_t)bytes[3 * p + 2];
                    }
                }
                continue;
            }
            if (net) {                                     // placed macroblock: one branch per row of 4 pixels
                const float* nrow = net + (size_t)yy * (iw * S) * 3;
                float nv[12];
                if (turned) {                              // output (yy, gx + p) <- block (gx + p, yy)
#pragma unroll
                    for (int p = 0; p < 4; ++p) {
                        const float* t = net + ((size_t)(gx + p) * (iw * S) + yy) * 3;
                        nv[3 * p] = t[0]; nv[3 * p + 1] = t[1]; nv[3 * p + 2] = t[2];
                    }
                } else if constexpr (S % 4 == 0) {         // 48-byte runs start 16-byte aligned
                    const float4 a0 = ((const float4*)nrow)[0], a1 = ((const float4*)nrow)[1], a2 = ((const float4*)nrow)[2];
                    nv[0] = a0.x; nv[1] = a0.y; nv[2] = a0.z; nv[3] = a0.w; nv[4] = a1.x; nv[5] = a1.y;
                    nv[6] = a1.z; nv[7] = a1.w; nv[8] = a2.x; nv[9] = a2.y; nv[10] = a2.z; nv[11] = a2.w;
                } else {
#pragma unroll
                    for (int k = 0; k < 12; ++k) nv[k] = nrow[k];
                }
                float ev[12];
#pragma unroll
                for (int k = 0; k < 12; ++k) {
                    const float e = fminf(fmaxf(__fadd_rn(q255[bytes[k]], nv[k]), 0.0f), 1.0f);
                    ev[k] = e;
                    bytes[k] = (uint32_t)__fadd_rn(__fmul_rn(e, 255.0f), 0.5f);   // >= 0: truncation = floor
                }
                if (sel) {
                    float* srow = sel + (((size_t)slot * B + yy) * B + gx) * 3;
#pragma unroll
                    for (int k = 0; k < 12; ++k) srow[k] = ev[k];
                }
            }
            uint32_t* o = (uint32_t*)(dst + (size_t)yy * HW * 3);
            const uint32_t w0 = bytes[0] | (bytes[1] << 8) | (bytes[2] << 16) | (bytes[3] << 24);
            const uint32_t w1 = bytes[4] | (bytes[5] << 8) | (bytes[6] << 16) | (bytes[7] << 24);
            const uint32_t w2 = bytes[8] | (bytes[9] << 8) | (bytes[10] << 16) | (bytes[11] << 24);
            o[0] = w0; o[1] = w1; o[2] = w2;
        }
#pragma unroll
        for (int k = 0; k < 6; ++k) { h0[k] = h1[k]; h1[k] = h2[k]; }
    }
}

__global__ __launch_bounds__(256) void k_fill_i32(int32_t* __restrict__ p, int32_t v, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
}

void rh_fill_i32(rh_ctx* ctx, int32_t* p, int32_t v, size_t n)
{
    const int nb = (int)((n + 255) / 256 < 1024 ? (n + 255) / 256 : 1024);
    hipLaunchKernelGGL(k_fill_i32, dim3(nb ? nb : 1), dim3(256), 0, ctx->stream, p, v, n);
}

rh_status rh_launch_unpack(rh_ctx* ctx, const float* enh, int n_img, int ih, int iw,
                           const rh_mbplace* places, const uint32_t* n_places,
                           const uint8_t* lr, int F, uint8_t* hr, float* sel)
{
    const uint32_t total = (uint32_t)ctx->per * F;
    rh_prof_scope ps(ctx, RH_PROF_UNPACK, 1);
    const int S = ctx->cfg.net.scale;
    const bool cut = ctx->cfg.frame_w % RH_MB || ctx->cfg.frame_h % RH_MB || ((ctx->cfg.frame_w * S * 3) & 3);
#define LAUNCH_UNPACK(SC)                                                                                       \
    do { if (cut) LAUNCH_UNPACK_E(SC, true); else LAUNCH_UNPACK_E(SC, false); } while (0)
#define LAUNCH_UNPACK_E(SC, E)                                                                                  \
    hipLaunchKernelGGL((k_unpack<SC, E>), dim3((ctx->mbw + (64 / (4 * SC)) - 1) / (64 / (4 * SC)), ctx->mbh, F), dim3(256), 0, \
                       ctx->stream, lr, ctx->cfg.frame_h, ctx->cfg.frame_w, ctx->mbw, enh, n_img, ih, iw, places,  \
                       n_places, total, hr, sel)
    if (S == 1) LAUNCH_UNPACK(1); else if (S == 2) LAUNCH_UNPACK(2); else if (S == 3) LAUNCH_UNPACK(3); else LAUNCH_UNPACK(4);
#undef LAUNCH_UNPACK
#undef LAUNCH_UNPACK_E
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

rh_status rh_launch_identity_places(rh_ctx* ctx, int F, rh_mbplace* places, uint32_t* n_places)
{
    const uint32_t total = (uint32_t)ctx->per * F;
    hipLaunchKernelGGL(k_identity_places, dim3((total + 255) / 256), dim3(256), 0, ctx->stream, places, n_places,
                       ctx->mbw, ctx->per, total);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

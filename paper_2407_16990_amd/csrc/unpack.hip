// Paste (Sec. 3.3.3) fused with the bilinear base IN(.) of the problem statement
// (Sec. 3.2.1): one pass writes every high-resolution pixel exactly once.  For a placed
// macroblock the pixel is clamp(base/255 + net) quantised, otherwise the base itself.
#include "rh_internal.h"

__global__ __launch_bounds__(256) void k_fill_i32(int32_t* __restrict__ p, int32_t v, size_t n)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) p[i] = v;
}

__global__ __launch_bounds__(256) void k_slot_scatter(const rh_mbplace* __restrict__ places,
                                                      const uint32_t* __restrict__ n_places, uint32_t cap,
                                                      int32_t* __restrict__ slot_of_mb)
{
    const uint32_t n = min(*n_places, cap);
    for (uint32_t i = blockIdx.x * 256u + threadIdx.x; i < n; i += gridDim.x * 256u) {
        const uint32_t g = places[i].mb_id;
        if (g < cap) slot_of_mb[g] = (int32_t)i;
    }
}

__global__ __launch_bounds__(256) void k_identity_places(rh_mbplace* __restrict__ places, uint32_t* __restrict__ n_places,
                                                         int mbw, int per, uint32_t total)
{
    const uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g == 0) *n_places = total;
    if (g >= total) return;
    const uint32_t f = g / per, in = g % per;
    rh_mbplace p;
    p.mb_id = g; p.box = f; p.bin = (uint16_t)f; p.px = (uint16_t)(RH_MB * (in % mbw)); p.py = (uint16_t)(RH_MB * (in / mbw)); p.pad = 0;
    places[g] = p;
}

// One workgroup per macroblock: (16s x 16s) output pixels from an 18 x 18 input tile in LDS.
// Each thread produces runs of 4 pixels = 12 bytes.
__global__ __launch_bounds__(256) void k_unpack(const uint8_t* __restrict__ lr, int H, int W, int s,
                                                const float* __restrict__ enh, int n_img, int ih, int iw,
                                                const rh_mbplace* __restrict__ places,
                                                const int32_t* __restrict__ slot_of_mb,
                                                uint8_t* __restrict__ hr, float* __restrict__ sel)
{
    __shared__ uint8_t tile[18][18][3];
    const int mx = blockIdx.x, my = blockIdx.y, f = blockIdx.z, tid = threadIdx.x;
    const int mbw = gridDim.x, mbh = gridDim.y;
    const uint8_t* src = lr + (size_t)f * H * W * 3;
    for (int i = tid; i < 18 * 18 * 3; i += 256) {
        const int c = i % 3, px = (i / 3) % 18, py = i / 54;
        const int y = min(max(RH_MB * my - 1 + py, 0), H - 1), x = min(max(RH_MB * mx - 1 + px, 0), W - 1);
        tile[py][px][c] = src[((size_t)y * W + x) * 3 + c];
    }
    const uint32_t g = ((uint32_t)f * mbh + my) * mbw + mx;
    const int slot = slot_of_mb[g];
    const float* net = nullptr;
    if (slot >= 0) {
        const rh_mbplace p = places[slot];
        if (p.bin != RH_NO_BIN && p.bin < n_img && p.px + RH_MB <= iw && p.py + RH_MB <= ih)
            net = enh + (((size_t)p.bin * (ih * s) + (size_t)p.py * s) * (iw * s) + (size_t)p.px * s) * 3;
    }
    __syncthreads();
    const int B = RH_MB * s, D = 2 * s, gpr = B / 4, ngrp = gpr * B;
    const int HW = W * s;
    uint8_t* dst = hr + (((size_t)f * H * s + (size_t)my * B) * HW + (size_t)mx * B) * 3;
    for (int grp = tid; grp < ngrp; grp += 256) {
        const int yy = grp / gpr, x4 = (grp - yy * gpr) * 4;
        // vertical taps: source row = (2Y+1-s)/(2s) relative to the tile (tile row 0 = 16my-1)
        const int ny = 2 * yy + 1 - s + D;                // shifted by one input row, always >= 0
        const int ty = ny / D, wy1 = ny - ty * D, wy0 = D - wy1;
        uint32_t bytes[12];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int nx = 2 * (x4 + p) + 1 - s + D;
            const int tx = nx / D, wx1 = nx - tx * D, wx0 = D - wx1;
#pragma unroll
            for (int c = 0; c < 3; ++c) {
                const int acc = wy0 * (wx0 * tile[ty][tx][c] + wx1 * tile[ty][tx + 1][c]) +
                                wy1 * (wx0 * tile[ty + 1][tx][c] + wx1 * tile[ty + 1][tx + 1][c]);
                uint32_t base = (uint32_t)(acc + D * D / 2) / (uint32_t)(D * D);
                if (net) {
                    const float nv = net[((size_t)yy * (iw * s) + x4 + p) * 3 + c];
                    float e = __fadd_rn(__fdiv_rn((float)base, 255.0f), nv);
                    e = fminf(fmaxf(e, 0.0f), 1.0f);
                    if (sel) sel[(((size_t)slot * B + yy) * B + x4 + p) * 3 + c] = e;
                    base = (uint32_t)floorf(__fadd_rn(__fmul_rn(e, 255.0f), 0.5f));
                }
                bytes[p * 3 + c] = base;
            }
        }
        uint32_t* o = (uint32_t*)(dst + ((size_t)yy * HW + x4) * 3);
        o[0] = bytes[0] | (bytes[1] << 8) | (bytes[2] << 16) | (bytes[3] << 24);
        o[1] = bytes[4] | (bytes[5] << 8) | (bytes[6] << 16) | (bytes[7] << 24);
        o[2] = bytes[8] | (bytes[9] << 8) | (bytes[10] << 16) | (bytes[11] << 24);
    }
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
    const int nb = (int)min((total + 255u) / 256u, 1024u);
    rh_prof_scope ps(ctx, RH_PROF_UNPACK, 3);
    rh_fill_i32(ctx, ctx->slot_of_mb, -1, (size_t)total);
    hipLaunchKernelGGL(k_slot_scatter, dim3(nb), dim3(256), 0, ctx->stream, places, n_places, total, ctx->slot_of_mb);
    hipLaunchKernelGGL(k_unpack, dim3(ctx->mbw, ctx->mbh, F), dim3(256), 0, ctx->stream, lr, ctx->cfg.frame_h,
                       ctx->cfg.frame_w, ctx->cfg.net.scale, enh, n_img, ih, iw, places, ctx->slot_of_mb, hr, sel);
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

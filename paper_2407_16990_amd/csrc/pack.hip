// Stitching (Sec. 3.3.3): copy every placed box, with its halo, from its frame into its bin.
// Bins are zero outside the boxes and where a halo leaves the frame.
#include "rh_internal.h"

// Zero bins [0, n_bins).  bin_vec = 16-byte vectors per bin.
__global__ __launch_bounds__(256) void k_bins_zero(uint4* __restrict__ bins, const uint32_t* __restrict__ counts,
                                                   size_t bin_vec)
{
    const size_t n = (size_t)counts[1] * bin_vec;
    const uint4 z = make_uint4(0, 0, 0, 0);
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) bins[i] = z;
}

// A work unit is an 8-row band of one box (as stored in the bin); workgroups stride over the units, each wave copies
// 2 rows, lanes run along the row's bytes (contiguous in both the frame and the bin).  Box
// rectangles of one bin are disjoint, so no two units write the same byte.
__global__ __launch_bounds__(256) void k_gather(const uint8_t* __restrict__ frames, const rh_box* __restrict__ boxes,
                                                const uint32_t* __restrict__ counts, int H, int W, int halo, int S,
                                                int bands, uint8_t* __restrict__ bins)
{
    const uint32_t n_units = counts[0] * (uint32_t)bands;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (uint32_t u = blockIdx.x; u < n_units; u += gridDim.x) {
        const rh_box b = boxes[u / bands];
        if (b.bin == RH_NO_BIN) continue;
        const int bw = RH_MB * b.wmb + 2 * halo, bh = RH_MB * b.hmb + 2 * halo, row_bytes = bw * 3;
        const int sx0 = RH_MB * b.mbx0 - halo, sy0 = RH_MB * b.mby0 - halo;
        const int x_lo = max(0, -sx0) * 3, x_hi = min(bw, W - sx0) * 3;   // in-frame byte range of a row
        const uint8_t* src = frames + (size_t)b.frame * H * W * 3;
        uint8_t* dst = bins + ((size_t)b.bin * S + b.by) * S * 3 + (size_t)b.bx * 3;
        if (b.rot) {
            // turned box: bin row i holds box column i, so a row's bytes come from one source
            // column (strided reads; turned boxes are the exception)
#pragma unroll
            for (int rr = 0; rr < 2; ++rr) {
                const int i = (u % bands) * 8 + wave * 2 + rr;     // bin row = box column
                if (i >= bw) continue;
                const int sx = sx0 + i;
                uint8_t* drow = dst + (size_t)i * S * 3;
                for (int c = lane; c < bh * 3; c += 64) {
                    const int j = c / 3, ch = c - 3 * j, sy = sy0 + j;
                    drow[c] = (sx >= 0 && sx < W && sy >= 0 && sy < H) ? src[((size_t)sy * W + sx) * 3 + ch] : (uint8_t)0;
                }
            }
            continue;
        }
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const int j = (u % bands) * 8 + wave * 2 + rr;
            if (j >= bh) continue;
            const int sy = sy0 + j;
            const bool row_in = sy >= 0 && sy < H;
            const uint8_t* srow = src + ((long)sy * W + sx0) * 3;
            uint8_t* drow = dst + (size_t)j * S * 3;
            for (int c = lane; c < row_bytes; c += 64) drow[c] = (row_in && c >= x_lo && c < x_hi) ? srow[c] : (uint8_t)0;
        }
    }
}

rh_status rh_launch_gather(rh_ctx* ctx, const uint8_t* frames, int F, const rh_box* boxes,
                           const uint32_t* counts, uint8_t* bins)
{
    (void)F;
    const int S = ctx->cfg.bin_size;
    const size_t bin_vec = (size_t)S * S * 3 / 16;
    rh_prof_scope ps(ctx, RH_PROF_GATHER, 2);
    hipLaunchKernelGGL(k_bins_zero, dim3(1024), dim3(256), 0, ctx->stream, (uint4*)bins, counts, bin_vec);
    const int bands = (RH_MB * ctx->T + 2 * ctx->cfg.halo + 7) / 8;
    hipLaunchKernelGGL(k_gather, dim3(4096), dim3(256), 0, ctx->stream, frames, boxes, counts, ctx->cfg.frame_h,
                       ctx->cfg.frame_w, ctx->cfg.halo, S, bands, bins);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

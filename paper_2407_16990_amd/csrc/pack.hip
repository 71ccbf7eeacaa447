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

// Workgroups stride over the boxes; a box's rows are contiguous byte runs in both the frame
// and the bin.  Box rectangles of one bin are disjoint, so no two workgroups write one byte.
__global__ __launch_bounds__(256) void k_gather(const uint8_t* __restrict__ frames, const rh_box* __restrict__ boxes,
                                                const uint32_t* __restrict__ counts, int H, int W, int halo, int S,
                                                uint8_t* __restrict__ bins)
{
    const uint32_t n = counts[0];
    for (uint32_t bi = blockIdx.x; bi < n; bi += gridDim.x) {
        const rh_box b = boxes[bi];
        if (b.bin == RH_NO_BIN) continue;
        const int bw = RH_MB * b.wmb + 2 * halo, bh = RH_MB * b.hmb + 2 * halo, row_bytes = bw * 3;
        const int sx0 = RH_MB * b.mbx0 - halo, sy0 = RH_MB * b.mby0 - halo;
        const uint8_t* src = frames + (size_t)b.frame * H * W * 3;
        uint8_t* dst = bins + ((size_t)b.bin * S + b.by) * S * 3 + (size_t)b.bx * 3;
        const int x_lo = max(0, -sx0) * 3, x_hi = min(bw, W - sx0) * 3;   // in-frame byte range of a row
        for (int idx = threadIdx.x; idx < bh * row_bytes; idx += 256) {
            const int j = idx / row_bytes, c = idx - j * row_bytes;
            const int sy = sy0 + j;
            uint8_t v = 0;
            if (sy >= 0 && sy < H && c >= x_lo && c < x_hi) v = src[((long)sy * W + sx0) * 3 + c];
            dst[(size_t)j * S * 3 + c] = v;
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
    hipLaunchKernelGGL(k_gather, dim3(2048), dim3(256), 0, ctx->stream, frames, boxes, counts, ctx->cfg.frame_h,
                       ctx->cfg.frame_w, ctx->cfg.halo, S, bins);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

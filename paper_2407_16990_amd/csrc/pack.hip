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

// A work unit is a band of 4 * GATHER_RPW rows of one box (as stored in the bin); workgroups stride over the
// units, each wave copies GATHER_RPW rows, lanes run along the row's bytes (contiguous in both the frame
// and the bin).  Box rectangles of one bin are disjoint, so no two units write the same byte.
#ifndef GATHER_RPW
#define GATHER_RPW 2
#endif
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
            for (int rr = 0; rr < GATHER_RPW; ++rr) {
                const int i = (u % bands) * (4 * GATHER_RPW) + wave * GATHER_RPW + rr;     // bin row = box column
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
        // Upright box: the band's rows go out as aligned 4-byte stores (plus up to 3 single bytes at
        // either end of a row).  Source and destination are misaligned against each other by an
        // arbitrary amount, so a destination word is funnelled out of the two aligned source words
        // that hold its bytes; each of those contains at least one byte of the row, hence lies in
        // mapped memory.  Words that straddle the frame's left or right edge are put together byte
        // by byte (bytes outside the frame are zero).  The words of the whole band are dealt to the
        // 256 threads, and a thread requests all of its words before it stores the first: the
        // kernel lives on the number of loads in flight.
        const int j0 = (u % bands) * (4 * GATHER_RPW), nrow = min(4 * GATHER_RPW, bh - j0);
        if (nrow <= 0) continue;
        const int head = (int)((4u - (unsigned)((uintptr_t)dst & 3u)) & 3u);     // the same for every row: the row pitch is a multiple of 4
        const int nd = (row_bytes - head) >> 2, tail0 = head + 4 * nd, nends = head + (row_bytes - tail0);
        const int tid = threadIdx.x;
        if (tid < nrow * nends) {                                                 // the few bytes at the rows' ends
            const int r = tid / nends, e = tid - r * nends, c = e < head ? e : tail0 + (e - head);
            const int sy = sy0 + j0 + r;
            const bool ok = sy >= 0 && sy < H && c >= x_lo && c < x_hi;
            dst[(size_t)(j0 + r) * S * 3 + c] = ok ? src[((long)sy * W + sx0) * 3 + c] : (uint8_t)0;
        }
        constexpr int WPT = 3;                                                    // words per thread and pass
        const int total = nrow * nd;
        for (int t0 = 0; t0 < total; t0 += WPT * 256) {
            uint32_t lo[WPT], hi[WPT]; int off[WPT]; unsigned sh[WPT]; bool funnel[WPT];
#pragma unroll
            for (int k = 0; k < WPT; ++k) {
                const int t = t0 + k * 256 + tid;
                funnel[k] = false; lo[k] = 0; hi[k] = 0; sh[k] = 0; off[k] = 0;
                if (t < total) {
                    const int r = t / nd, i = t - r * nd, c = head + 4 * i, sy = sy0 + j0 + r;
                    off[k] = (j0 + r) * S * 3 + c;
                    const bool row_in = sy >= 0 && sy < H;
                    const uint8_t* sp = src + ((long)sy * W + sx0) * 3 + c;
                    if (row_in && c >= x_lo && c + 4 <= x_hi) {
                        const uintptr_t sa = (uintptr_t)sp;
                        const uint32_t* p = (const uint32_t*)(sa & ~(uintptr_t)3);
                        sh[k] = (unsigned)(sa & 3);
                        lo[k] = p[0];
                        if (sh[k]) hi[k] = p[1];
                        funnel[k] = true;
                    } else {                                  // outside the frame, or across its edge: rare, stored at once
                        uint32_t w = 0;
                        if (row_in) {
#pragma unroll
                            for (int q = 0; q < 4; ++q)
                                if (c + q >= x_lo && c + q < x_hi) w |= (uint32_t)sp[q] << (8 * q);
                        }
                        *(uint32_t*)(dst + off[k]) = w;
                    }
                }
            }
#pragma unroll
            for (int k = 0; k < WPT; ++k)
                if (funnel[k]) *(uint32_t*)(dst + off[k]) = sh[k] ? __builtin_amdgcn_alignbyte(hi[k], lo[k], sh[k]) : lo[k];
        }
    }
}

// Exact-border mode.  Sets to zero, in an activation tensor [N][S*res][S*res] of px_bytes-byte
// pixels, the part of every placed box whose source pixels lie outside the frame.  Unit = 8-row
// band of a box as stored in the bin; a wave takes 2 stored rows.  Per stored row the outside
// part is the whole row (the source row - or, for a turned box, column - is outside) or a run at
// each end; the runs are cleared with 16-byte stores (px_bytes is a multiple of 16).
__global__ __launch_bounds__(256) void k_zero_outside(uint8_t* __restrict__ act, int px_bytes, int res,
                                                      const rh_box* __restrict__ boxes, const uint32_t* __restrict__ counts,
                                                      int n_img, const uint32_t* __restrict__ n_valid, int H, int W,
                                                      int halo, int S, int bands)
{
    const uint32_t n_units = counts[0] * (uint32_t)bands;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nv = n_valid ? min((int)*n_valid, n_img) : n_img;
    const size_t row_pitch = (size_t)S * res * px_bytes;
    for (uint32_t u = blockIdx.x; u < n_units; u += gridDim.x) {
        const rh_box b = boxes[u / bands];
        if (b.bin == RH_NO_BIN || (int)b.bin >= nv) continue;
        const int bw = RH_MB * b.wmb + 2 * halo, bh = RH_MB * b.hmb + 2 * halo;
        const int sx0 = RH_MB * b.mbx0 - halo, sy0 = RH_MB * b.mby0 - halo;
        if (sx0 >= 0 && sy0 >= 0 && sx0 + bw <= W && sy0 + bh <= H) continue;      // box entirely inside the frame
        // stored rows run along the box's rows (upright) or columns (turned)
        const int n_rows = b.rot ? bw : bh, n_cols = b.rot ? bh : bw;
        if (b.bx + n_cols > S || b.by + n_rows > S) continue;                      // not a box of this geometry: never write outside the bin
        const int r0 = b.rot ? sx0 : sy0, rlim = b.rot ? W : H;                    // source coordinate of stored row 0, its limit
        const int c0s = b.rot ? sy0 : sx0, clim = b.rot ? H : W;                   // same for stored columns
        const int lo_end = min(n_cols, max(0, -c0s)), hi_beg = max(0, min(n_cols, clim - c0s));
#pragma unroll
        for (int rr = 0; rr < 2; ++rr) {
            const int j = (u % bands) * 8 + wave * 2 + rr;
            if (j >= n_rows) continue;
            const bool row_out = r0 + j < 0 || r0 + j >= rlim;
            // runs of stored columns to clear: [0, e0) and [b1, n_cols)
            const int e0 = row_out ? n_cols : lo_end, b1 = row_out ? n_cols : hi_beg;
            for (int dy = 0; dy < res; ++dy) {
                uint8_t* row = act + ((size_t)b.bin * S * res + (size_t)(b.by + j) * res + dy) * row_pitch + (size_t)b.bx * res * px_bytes;
                const int n0 = e0 * res * px_bytes / 16, s1 = b1 * res * px_bytes / 16, n1 = n_cols * res * px_bytes / 16;
                for (int c = lane; c < n0; c += 64) ((uint4*)row)[c] = make_uint4(0, 0, 0, 0);
                for (int c = s1 + lane; c < n1; c += 64) ((uint4*)row)[c] = make_uint4(0, 0, 0, 0);
            }
        }
    }
}

rh_status rh_zero_outside(rh_ctx* ctx, void* act, int px_bytes, int res, int N, const uint32_t* n_valid)
{
    if (!ctx->bz_boxes) return RH_OK;
    if (px_bytes % 16) RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "exact-border mode needs pixels of a multiple of 16 bytes, got %d", px_bytes);
    const int bands = (RH_MB * ctx->T + 2 * ctx->cfg.halo + 7) / 8;
    hipLaunchKernelGGL(k_zero_outside, dim3(2048), dim3(256), 0, ctx->stream, (uint8_t*)act, px_bytes, res, ctx->bz_boxes,
                       ctx->bz_counts, N, n_valid, ctx->cfg.frame_h, ctx->cfg.frame_w, ctx->cfg.halo, ctx->cfg.bin_size, bands);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

rh_status rh_launch_gather(rh_ctx* ctx, const uint8_t* frames, int F, const rh_box* boxes,
                           const uint32_t* counts, uint8_t* bins)
{
    (void)F;
    const int S = ctx->cfg.bin_size;
    const size_t bin_vec = (size_t)S * S * 3 / 16;
    rh_prof_scope ps(ctx, RH_PROF_GATHER, 2);
    hipLaunchKernelGGL(k_bins_zero, dim3(1024), dim3(256), 0, ctx->stream, (uint4*)bins, counts, bin_vec);
    const int bands = (RH_MB * ctx->T + 2 * ctx->cfg.halo + 4 * GATHER_RPW - 1) / (4 * GATHER_RPW);
    hipLaunchKernelGGL(k_gather, dim3(4096), dim3(256), 0, ctx->stream, frames, boxes, counts, ctx->cfg.frame_h,
                       ctx->cfg.frame_w, ctx->cfg.halo, S, bands, bins);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

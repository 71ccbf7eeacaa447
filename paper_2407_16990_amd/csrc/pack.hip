// Stitching (Sec. 3.3.3): copy every placed box, with its halo, from its frame into its bin.
// Bins are zero outside the boxes and where a halo leaves the frame.
#include "rh_internal.h"

// One launch writes every byte of bins [0, n_bins) exactly once.  A work unit is a band of RB rows
// of one bin, put together in LDS and written out as whole 16-byte vectors (the band is one
// contiguous piece of the bin tensor):
//   1. the band's LDS image is cleared and the box list is scanned for boxes of this bin that
//      reach into the band (a 2-byte field per box; the few that match are listed in LDS);
//   2. every listed box adds its pixels: the frame's bytes are fetched as aligned 4-byte words and
//      shifted into place (frame and bin positions are misaligned against each other by an
//      arbitrary amount), bytes outside the frame or outside the box are masked to zero, and the
//      word is OR-ed into the cleared image, so boxes that meet inside one word compose;
//   3. the image goes to the bin.
// Box rectangles of one bin are disjoint, so the result does not depend on the order of the boxes.
#define GATHER_LIST 64

__device__ __forceinline__ uint32_t byte_mask(int lo_cut, int hi_cut)      // bytes [lo_cut, hi_cut) of a word, cuts in 0..4
{
    const uint32_t below_hi = hi_cut >= 4 ? 0xFFFFFFFFu : ((1u << (8 * hi_cut)) - 1u);
    const uint32_t below_lo = lo_cut >= 4 ? 0xFFFFFFFFu : ((1u << (8 * lo_cut)) - 1u);
    return below_hi & ~below_lo;
}

// Adds the part of box b that lies in rows [y0, y0 + rows) of its bin to the band image.
__device__ __forceinline__ void gather_box(const rh_box& b, const uint8_t* __restrict__ frames, int H, int W, int halo,
                                           int S, int y0, int rows, uint32_t* img)
{
    const int bw = RH_MB * b.wmb + 2 * halo, bh = RH_MB * b.hmb + 2 * halo;
    const int sx0 = RH_MB * b.mbx0 - halo, sy0 = RH_MB * b.mby0 - halo;
    const int n_rows = b.rot ? bw : bh, n_cols = b.rot ? bh : bw;          // as stored in the bin
    const int j0 = max(0, y0 - (int)b.by), j1 = min(n_rows, y0 + rows - (int)b.by);
    if (j1 <= j0) return;
    const uint8_t* src = frames + (size_t)b.frame * H * W * 3;
    const int L = n_cols * 3, pitch_w = S * 3 / 4;                         // row length in bytes; band row pitch in words
    const int dofs = (((int)b.by + j0 - y0) * S + (int)b.bx) * 3;          // byte offset of the first stored row in the image
    const int head = dofs & 3, ndw = (head + L + 3) >> 2, items = (j1 - j0) * ndw;
    for (int t = threadIdx.x; t < items; t += 256) {
        const int r = t / ndw, kk = t - r * ndw, j = j0 + r;
        const int c = 4 * kk - head;                                       // row byte held by the word's first byte (may be < 0)
        uint32_t v = 0;
        if (b.rot) {
            // turned box: stored row j holds box column j, so its bytes come from one source column
            const int sx = sx0 + j;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int cc = c + q;
                if (cc < 0 || cc >= L) continue;
                const int jj = cc / 3, ch = cc - 3 * jj, sy = sy0 + jj;
                if (sx >= 0 && sx < W && sy >= 0 && sy < H) v |= (uint32_t)src[((size_t)sy * W + sx) * 3 + ch] << (8 * q);
            }
        } else {
            const int sy = sy0 + j;
            if (sy < 0 || sy >= H) continue;
            const int vb = max(0, -sx0) * 3, ve = min(bw, W - sx0) * 3;    // in-frame bytes of a row
            const int lo_cut = min(max(vb - c, 0), 4), hi_cut = min(max(ve - c, 0), 4);
            if (hi_cut <= lo_cut) continue;
            const uintptr_t sa = (uintptr_t)(src + ((long)sy * W + sx0) * 3) + (long)c;
            const uint32_t* al = (const uint32_t*)(sa & ~(uintptr_t)3);
            const int sh = (int)(sa & 3);
            // an aligned word is fetched only if it holds one of the wanted bytes (hence lies in mapped memory)
            uint32_t lo = 0, hi = 0;
            if (4 - sh > lo_cut) lo = al[0];
            if (sh && 4 - sh < hi_cut) hi = al[1];
            v = (sh ? __builtin_amdgcn_alignbyte(hi, lo, sh) : lo) & byte_mask(lo_cut, hi_cut);
        }
        if (v) atomicOr(&img[(dofs >> 2) + r * pitch_w + kk], v);
    }
}

__global__ __launch_bounds__(256) void k_gather(const uint8_t* __restrict__ frames, const rh_box* __restrict__ boxes,
                                                const uint32_t* __restrict__ counts, int H, int W, int halo, int S,
                                                int RB, uint8_t* __restrict__ bins)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t img[];         // RB * S * 3 bytes
    __shared__ uint32_t s_list[GATHER_LIST];
    __shared__ uint32_t s_cnt;
    const uint32_t n_boxes = counts[0], n_bins = counts[1];
    const int nb = (S + RB - 1) / RB;                                      // bands per bin
    // A unit is a run of bpu bands of one bin; the box list is scanned once per unit.  Small batches
    // take one band per unit (enough units to occupy the chip), large ones a whole bin.
    const int bpu = (uint64_t)n_bins * (uint64_t)nb <= 2048u ? 1 : nb;
    const int upb = (nb + bpu - 1) / bpu;                                  // units per bin
    const int tid = threadIdx.x;
    for (uint32_t u = blockIdx.x; u < n_bins * (uint32_t)upb; u += gridDim.x) {
        const uint32_t bin = u / upb;
        const int ya = (int)(u - bin * upb) * bpu * RB, yb = min(S, ya + bpu * RB);   // rows [ya, yb) of the bin
        if (tid == 0) s_cnt = 0;
        __syncthreads();
        for (uint32_t i = tid; i < n_boxes; i += 256) {
            if (boxes[i].bin != bin) continue;
            const rh_box b = boxes[i];
            const int n_rows = b.rot ? RH_MB * b.wmb + 2 * halo : RH_MB * b.hmb + 2 * halo;
            if ((int)b.by < yb && (int)b.by + n_rows > ya) {
                const uint32_t k = atomicAdd(&s_cnt, 1u);
                if (k < GATHER_LIST) s_list[k] = i;
            }
        }
        for (int y0 = ya; y0 < yb; y0 += RB) {
            const int rows = min(RB, yb - y0);
            const int n_vec = rows * S * 3 / 16;                           // S is a multiple of 4 and so is rows
            for (int i = tid; i < n_vec; i += 256) ((uint4*)img)[i] = make_uint4(0, 0, 0, 0);
            __syncthreads();                                               // image cleared, list complete
            const uint32_t cnt = s_cnt;                                    // uniform over the workgroup
            if (cnt <= GATHER_LIST) {
                for (uint32_t k = 0; k < cnt; ++k) gather_box(boxes[s_list[k]], frames, H, W, halo, S, y0, rows, img);
            } else {
                // more boxes reach into these rows than the list holds (tiny boxes in very wide bins):
                // go through all boxes one after the other
                for (uint32_t i = 0; i < n_boxes; ++i) {
                    const rh_box b = boxes[i];
                    if (b.bin == bin) gather_box(b, frames, H, W, halo, S, y0, rows, img);
                }
            }
            __syncthreads();
            uint4* dst = (uint4*)(bins + ((size_t)bin * S + y0) * S * 3);
            for (int i = tid; i < n_vec; i += 256) dst[i] = ((const uint4*)img)[i];
            __syncthreads();
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
    if ((uintptr_t)bins & 15) RH_FAIL(ctx, RH_E_INVALID, "rh_pack: bins must be 16-byte aligned");
    // rows per band: a multiple of 4 (whole 16-byte vectors), about 6 KB of LDS image, at most 48 KB
    int RB = (6 * 1024 / (S * 3)) & ~3;
    RB = RB < 4 ? 4 : (RB > 32 ? 32 : RB);
    const size_t lds = (size_t)RB * S * 3;
    static bool attr_done[RH_MAX_DEVICES] = {};
    if (!attr_done[ctx->device]) {
        RH_HIP(ctx, hipFuncSetAttribute((const void*)k_gather, hipFuncAttributeMaxDynamicSharedMemorySize, 48 * 1024));
        attr_done[ctx->device] = true;
    }
    const long units = (long)ctx->cfg.max_bins * ((S + RB - 1) / RB);
    const int grid = (int)(units < 4096 ? (units > 0 ? units : 1) : 4096);
    rh_prof_scope ps(ctx, RH_PROF_GATHER, 1);
    hipLaunchKernelGGL(k_gather, dim3(grid), dim3(256), lds, ctx->stream, frames, boxes, counts, ctx->cfg.frame_h,
                       ctx->cfg.frame_w, ctx->cfg.halo, S, RB, bins);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

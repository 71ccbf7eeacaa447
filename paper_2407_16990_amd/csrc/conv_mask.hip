// Box-masked enhance mode (Sec. 3.3.2: a packed bin is only partly occupied).
//
// A bin is cut into cells of RH_CELL_H x RH_CELL_W pixels - the half tile that is the unit of
// work of the 64-channel conv kernel - and a cell is live when a placed box (with its halo)
// shares a pixel with it.  The body convs compute the live cells only; every other cell of the
// three activation tensors they read is zero.  Three small launches per call:
//   k_cell_mark  : one thread per box sets the mark byte of every cell the box touches
//   k_cell_lists : one wave per bin turns the marks into the list of live cells (what the conv
//                  kernel walks) and the list of the others (what gets cleared), and clears the
//                  marks again
//   k_zero_cells : writes zeros over the other cells of the activation tensors
// The cells of one bin stay together in the lists (bins in the order their waves arrive), which
// keeps neighbouring tiles - the ones that share halo pixels - next to each other in the walk.
#include "rh_internal.h"

__global__ __launch_bounds__(256) void k_cell_mark(const rh_box* __restrict__ boxes, const uint32_t* __restrict__ counts,
                                                   int N, const uint32_t* __restrict__ n_valid, int halo, int cells_x,
                                                   int cells_y, uint8_t* __restrict__ mark, uint32_t* __restrict__ cnt)
{
    const uint32_t g = blockIdx.x * 256u + threadIdx.x;
    if (g == 0) { cnt[0] = 0; cnt[1] = 0; }
    const uint32_t n_boxes = counts[0];
    const int n_img = n_valid ? min((int)*n_valid, N) : N;
    for (uint32_t i = g; i < n_boxes; i += gridDim.x * 256u) {
        const rh_box b = boxes[i];
        if (b.bin == RH_NO_BIN || (int)b.bin >= n_img) continue;
        const int bw = RH_MB * b.wmb + 2 * halo, bh = RH_MB * b.hmb + 2 * halo;
        const int fw = b.rot ? bh : bw, fh = b.rot ? bw : bh;              // extent inside the bin
        const int cx0 = b.bx / RH_CELL_W, cx1 = min((b.bx + fw - 1) / RH_CELL_W, cells_x - 1);
        const int cy0 = b.by / RH_CELL_H, cy1 = min((b.by + fh - 1) / RH_CELL_H, cells_y - 1);
        for (int cy = cy0; cy <= cy1; ++cy)
            for (int cx = cx0; cx <= cx1; ++cx) mark[((size_t)b.bin * cells_y + cy) * cells_x + cx] = 1;
    }
}

__global__ __launch_bounds__(256) void k_cell_lists(int N, const uint32_t* __restrict__ n_valid, int cells_img, int cells_x,
                                                    uint8_t* __restrict__ mark, uint32_t* __restrict__ live,
                                                    uint32_t* __restrict__ dead, uint32_t* __restrict__ cnt)
{
    const int lane = threadIdx.x & 63, bin = blockIdx.x * 4 + (threadIdx.x >> 6);
    const int n_img = n_valid ? min((int)*n_valid, N) : N;
    if (bin >= n_img) return;                                  // whole waves leave
    uint8_t* m = mark + (size_t)bin * cells_img;
    uint32_t n_live = 0;
    for (int c0 = 0; c0 < cells_img; c0 += 64) {
        const bool on = c0 + lane < cells_img && m[c0 + lane] != 0;
        n_live += (uint32_t)__popcll(__ballot(on));
    }
    uint32_t base_l = 0, base_d = 0;
    if (lane == 0) { base_l = atomicAdd(&cnt[0], n_live); base_d = atomicAdd(&cnt[1], (uint32_t)cells_img - n_live); }
    base_l = (uint32_t)__shfl((int)base_l, 0); base_d = (uint32_t)__shfl((int)base_d, 0);
    for (int c0 = 0; c0 < cells_img; c0 += 64) {
        const bool in = c0 + lane < cells_img, on = in && m[c0 + lane] != 0;
        const unsigned long long bl = __ballot(on), bd = __ballot(in && !on);
        const unsigned long long below = (1ull << lane) - 1ull;
        const uint32_t id = RH_CELL_ENTRY(bin, (c0 + lane) / cells_x, (c0 + lane) % cells_x);
        if (on) live[base_l + (uint32_t)__popcll(bl & below)] = id;
        else if (in) dead[base_d + (uint32_t)__popcll(bd & below)] = id;
        if (on) m[c0 + lane] = 0;                              // marks are all zero between calls
        base_l += (uint32_t)__popcll(bl); base_d += (uint32_t)__popcll(bd);
    }
}

// act0..2: bf16 [N][H][W][64] (128 bytes per pixel); one workgroup clears one listed cell at a time
__global__ __launch_bounds__(256) void k_zero_cells(uint8_t* __restrict__ act0, uint8_t* __restrict__ act1,
                                                    uint8_t* __restrict__ act2, const uint32_t* __restrict__ dead,
                                                    const uint32_t* __restrict__ cnt, int H, int W)
{
    const uint32_t n_dead = cnt[1];
    const int px = threadIdx.x >> 3, piece = threadIdx.x & 7;
    for (uint32_t i = blockIdx.x; i < n_dead; i += gridDim.x) {
        const uint32_t id = dead[i];
        const int n = (int)(id >> 16);
        const int y0 = (int)((id >> 7) & 511u) * RH_CELL_H, x = (int)(id & 127u) * RH_CELL_W + px;
        if (x >= W) continue;
        for (int r = 0; r < RH_CELL_H && y0 + r < H; ++r) {
            const size_t off = (((size_t)n * H + (y0 + r)) * W + x) * 128 + piece * 16;
            *(uint4*)(act0 + off) = make_uint4(0, 0, 0, 0);
            *(uint4*)(act1 + off) = make_uint4(0, 0, 0, 0);
            *(uint4*)(act2 + off) = make_uint4(0, 0, 0, 0);
        }
    }
}

rh_status rh_mask_init(rh_ctx* ctx)
{
    const int S = ctx->cfg.bin_size;
    ctx->cells_x = (S + RH_CELL_W - 1) / RH_CELL_W; ctx->cells_y = (S + RH_CELL_H - 1) / RH_CELL_H;
    const size_t cap = (size_t)ctx->cfg.max_bins * ctx->cells_x * ctx->cells_y;
    RH_HIP(ctx, hipMalloc((void**)&ctx->cell_mark, cap + 16));
    RH_HIP(ctx, hipMemset(ctx->cell_mark, 0, cap + 16));
    RH_HIP(ctx, hipMalloc((void**)&ctx->cell_live, cap * 4 + 16));
    RH_HIP(ctx, hipMalloc((void**)&ctx->cell_dead, cap * 4 + 16));
    RH_HIP(ctx, hipMalloc((void**)&ctx->cell_cnt, 16));
    RH_HIP(ctx, hipMemset(ctx->cell_cnt, 0, 16));
    return RH_OK;
}

// Builds the cell lists of the bins of the masked call in progress and clears the other cells of
// the three [N][S][S][64] bf16 tensors.  Enqueue only.
rh_status rh_launch_cell_lists(rh_ctx* ctx, int N, const uint32_t* n_valid, void* act0, void* act1, void* act2)
{
    const int S = ctx->cfg.bin_size, cells_img = ctx->cells_x * ctx->cells_y;
    hipLaunchKernelGGL(k_cell_mark, dim3(64), dim3(256), 0, ctx->stream, ctx->mk_boxes, ctx->mk_counts, N, n_valid,
                       ctx->cfg.halo, ctx->cells_x, ctx->cells_y, ctx->cell_mark, ctx->cell_cnt);
    hipLaunchKernelGGL(k_cell_lists, dim3((N + 3) / 4), dim3(256), 0, ctx->stream, N, n_valid, cells_img, ctx->cells_x, ctx->cell_mark,
                       ctx->cell_live, ctx->cell_dead, ctx->cell_cnt);
    hipLaunchKernelGGL(k_zero_cells, dim3(1024), dim3(256), 0, ctx->stream, (uint8_t*)act0, (uint8_t*)act1, (uint8_t*)act2,
                       ctx->cell_dead, ctx->cell_cnt, S, S);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

// ---------------------------------------------------------------------------------------------
// Needed-region mode.  Only the pixels of placed macroblocks are ever pasted, and a conv output is
// read by the next conv within one pixel only, so layer by layer the part of a bin that can reach a
// pasted pixel shrinks: the conv whose output feeds the paste through r more pixels of reach needs
// to be right only within Chebyshev distance r of a placed macroblock.  For every cell the smallest
// such distance is computed once per call; list r holds the cells at distance <= r, r = 0 .. RH_NEED_RMAX,
// and every body conv (and the composed tail) walks the list of its own radius.  What lies outside
// is never read by anything that reaches a pasted pixel, so it is neither computed nor cleared.
//   k_need_mark  : one thread per placed macroblock lowers the distance of the cells around it
//   k_need_lists : one wave per bin: histogram of the distances -> one atomic per radius for the
//                  list bases -> ordered writes; the distances are reset for the next call
__device__ __forceinline__ void wave_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(256) void k_need_mark(const rh_mbplace* __restrict__ places, const uint32_t* __restrict__ counts,
                                                   uint32_t place_cap, int N, const uint32_t* __restrict__ n_valid, int S,
                                                   int cells_x, int cells_y, int rmax, uint32_t* __restrict__ dmin,
                                                   uint32_t* __restrict__ cnt)
{   // rmax: the largest radius any layer of this network asks for (<= RH_NEED_RMAX).  One wave per placed
    // macroblock, one lane per cell of the window around it: a lane's read and atomic depend on nothing else.
    const int lane = threadIdx.x & 63;
    const uint32_t wave = blockIdx.x * 4u + (threadIdx.x >> 6), n_waves = gridDim.x * 4u;
    if (blockIdx.x == 0 && threadIdx.x <= RH_NEED_RMAX) cnt[threadIdx.x] = 0;
    const uint32_t n_places = min(counts[3], place_cap);
    const int n_img = n_valid ? min((int)*n_valid, N) : N;
    for (uint32_t i = wave; i < n_places; i += n_waves) {
        const rh_mbplace p = places[i];
        if (p.bin == RH_NO_BIN || (int)p.bin >= n_img || (int)p.px + RH_MB > S || (int)p.py + RH_MB > S) continue;
        const int x0 = p.px, y0 = p.py;                        // the macroblock covers [x0, x0 + 15] x [y0, y0 + 15]
        const int cxa = max(0, x0 - rmax) / RH_CELL_W, cxb = min(cells_x - 1, (x0 + RH_MB - 1 + rmax) / RH_CELL_W);
        const int cya = max(0, y0 - rmax) / RH_CELL_H, cyb = min(cells_y - 1, (y0 + RH_MB - 1 + rmax) / RH_CELL_H);
        const int nx = cxb - cxa + 1, total = nx * (cyb - cya + 1);
        for (int t = lane; t < total; t += 64) {
            const int cy = cya + t / nx, cx = cxa + t % nx;
            const int gy = max(0, max(cy * RH_CELL_H - (y0 + RH_MB - 1), y0 - (cy * RH_CELL_H + RH_CELL_H - 1)));
            const int gx = max(0, max(cx * RH_CELL_W - (x0 + RH_MB - 1), x0 - (cx * RH_CELL_W + RH_CELL_W - 1)));
            const int d = max(gx, gy);                         // the cell is reached by a dilation of the macroblock by d pixels
            uint32_t* cell = &dmin[((size_t)p.bin * cells_y + cy) * cells_x + cx];
            // most cells already hold a smaller distance from a neighbouring macroblock: look before the atomic
            // (a stale read can only be too large, which costs an atomic, never a result)
            if (d <= rmax && *cell > (uint32_t)d) atomicMin(cell, (uint32_t)d);
        }
    }
}

__global__ __launch_bounds__(256) void k_need_lists(int N, const uint32_t* __restrict__ n_valid, int cells_img, int cells_x,
                                                    int rmax, uint32_t* __restrict__ dmin, uint32_t* __restrict__ lists, size_t cap,
                                                    uint32_t* __restrict__ cnt)
{
    __shared__ uint32_t s_hist[4][64];
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6, bin = blockIdx.x * 4 + w;
    const int n_img = n_valid ? min((int)*n_valid, N) : N;
    if (bin >= n_img) return;                                  // whole waves leave; nothing below synchronises across waves
    uint32_t* dm = dmin + (size_t)bin * cells_img;
    s_hist[w][lane] = 0;
    wave_fence();
    for (int c0 = 0; c0 < cells_img; c0 += 64) {
        const uint32_t d = c0 + lane < cells_img ? dm[c0 + lane] : 0xFFFFFFFFu;
        if (d <= RH_NEED_RMAX) atomicAdd(&s_hist[w][d], 1u);
    }
    wave_fence();
    uint32_t upto = 0;                                         // cells of this bin at distance <= lane
    for (int d = 0; d <= lane; ++d) upto += s_hist[w][d];
    uint32_t mybase = upto ? atomicAdd(&cnt[lane], upto) : 0u;        // lane r: where list r continues
    for (int c0 = 0; c0 < cells_img; c0 += 64) {
        const bool in = c0 + lane < cells_img;
        const uint32_t d = in ? dm[c0 + lane] : 0xFFFFFFFFu;
        const uint32_t id = RH_CELL_ENTRY(bin, (c0 + lane) / cells_x, (c0 + lane) % cells_x);
        const unsigned long long below = (1ull << lane) - 1ull;
        for (int r = 0; r <= rmax; ++r) {
            const unsigned long long m = __ballot(d <= (uint32_t)r);
            if (!m) continue;                                  // uniform
            const uint32_t base = (uint32_t)__builtin_amdgcn_readlane((int)mybase, r);
            if (d <= (uint32_t)r) lists[(size_t)r * cap + base + (uint32_t)__popcll(m & below)] = id;
            if (lane == r) mybase += (uint32_t)__popcll(m);
        }
        if (in && d != 0xFFFFFFFFu) dm[c0 + lane] = 0xFFFFFFFFu;    // all distances are "none" between calls
    }
}

// Scratch of the needed-region mode, allocated at the first call that uses it.
static rh_status need_alloc(rh_ctx* ctx)
{
    if (ctx->need_dmin) return RH_OK;
    const size_t cap = (size_t)ctx->cfg.max_bins * ctx->cells_x * ctx->cells_y;
    RH_HIP(ctx, hipMalloc((void**)&ctx->need_dmin, cap * 4 + 16));
    RH_HIP(ctx, hipMemset(ctx->need_dmin, 0xFF, cap * 4 + 16));
    RH_HIP(ctx, hipMalloc((void**)&ctx->need_lists, (size_t)(RH_NEED_RMAX + 1) * cap * 4 + 16));
    RH_HIP(ctx, hipMalloc((void**)&ctx->need_cnt, (RH_NEED_RMAX + 1) * 4));
    RH_HIP(ctx, hipMemset(ctx->need_cnt, 0, (RH_NEED_RMAX + 1) * 4));
    ctx->need_cap = cap;
    return RH_OK;
}

// Builds the per-radius cell lists of the needed-region call in progress.  Enqueue only (the first
// call allocates).
rh_status rh_launch_need_lists(rh_ctx* ctx, int N, const uint32_t* n_valid)
{
    rh_status st = need_alloc(ctx);
    if (st != RH_OK) return st;
    const int cells_img = ctx->cells_x * ctx->cells_y;
    const uint32_t place_cap = (uint32_t)ctx->cfg.max_frames * (uint32_t)ctx->per;
    const int rmax = ctx->nd_radii[0] < RH_NEED_RMAX ? ctx->nd_radii[0] : RH_NEED_RMAX;
    hipLaunchKernelGGL(k_need_mark, dim3(512), dim3(256), 0, ctx->stream, ctx->nd_places, ctx->nd_counts, place_cap, N, n_valid,
                       ctx->cfg.bin_size, ctx->cells_x, ctx->cells_y, rmax, ctx->need_dmin, ctx->need_cnt);
    hipLaunchKernelGGL(k_need_lists, dim3((N + 3) / 4), dim3(256), 0, ctx->stream, N, n_valid, cells_img, ctx->cells_x, rmax, ctx->need_dmin,
                       ctx->need_lists, ctx->need_cap, ctx->need_cnt);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

// Output radius of every layer of the needed-region mode: radii[0] the first conv, radii[1 .. nb] the
// nb bf16-output convs after it in execution order, radii[nb + 1] = 0 the layers after the body (their
// output is needed on the pasted pixels themselves).  The tail reaches `reach` low-resolution
// pixels into the body's output (composed upsampler + last conv: 2; a single last conv: 1) and
// every conv before it one more.  Returns nb, or -1 when the mode does not cover the network.
extern "C" int32_t rh_needed_radii(const rh_net_desc* net, int32_t per_layer_tail, int32_t* radii, int32_t cap)
{
    if (!net || !radii) return -1;
    int nb, reach;
    if (net->topology == RH_NET_EDSR) { if (per_layer_tail) return -1; nb = 2 * net->n_blocks + 1; reach = 2; }
    else if (net->topology == RH_NET_RES) { nb = 2 * net->n_blocks; reach = 1; }
    else if (net->topology == RH_NET_PLAIN) { nb = net->n_blocks - 2; reach = 1; }
    else return -1;
    if (nb < 0 || cap < nb + 2) return -1;
    radii[0] = reach + nb;
    for (int c = 0; c < nb; ++c) radii[1 + c] = reach + (nb - 1 - c);
    radii[nb + 1] = 0;
    return nb;
}

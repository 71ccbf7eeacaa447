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

__global__ __launch_bounds__(256) void k_cell_lists(int N, const uint32_t* __restrict__ n_valid, int cells_img,
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
        const uint32_t id = (uint32_t)bin * (uint32_t)cells_img + (uint32_t)(c0 + lane);
        if (on) live[base_l + (uint32_t)__popcll(bl & below)] = id;
        else if (in) dead[base_d + (uint32_t)__popcll(bd & below)] = id;
        if (on) m[c0 + lane] = 0;                              // marks are all zero between calls
        base_l += (uint32_t)__popcll(bl); base_d += (uint32_t)__popcll(bd);
    }
}

// act0..2: bf16 [N][H][W][64] (128 bytes per pixel); one workgroup clears one listed cell at a time
__global__ __launch_bounds__(256) void k_zero_cells(uint8_t* __restrict__ act0, uint8_t* __restrict__ act1,
                                                    uint8_t* __restrict__ act2, const uint32_t* __restrict__ dead,
                                                    const uint32_t* __restrict__ cnt, int H, int W, int cells_x, int cells_img)
{
    const uint32_t n_dead = cnt[1];
    const int px = threadIdx.x >> 3, piece = threadIdx.x & 7;
    for (uint32_t i = blockIdx.x; i < n_dead; i += gridDim.x) {
        const uint32_t id = dead[i];
        const int n = (int)(id / (uint32_t)cells_img), c = (int)(id % (uint32_t)cells_img);
        const int y0 = (c / cells_x) * RH_CELL_H, x = (c % cells_x) * RH_CELL_W + px;
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
    hipLaunchKernelGGL(k_cell_lists, dim3((N + 3) / 4), dim3(256), 0, ctx->stream, N, n_valid, cells_img, ctx->cell_mark,
                       ctx->cell_live, ctx->cell_dead, ctx->cell_cnt);
    hipLaunchKernelGGL(k_zero_cells, dim3(1024), dim3(256), 0, ctx->stream, (uint8_t*)act0, (uint8_t*)act1, (uint8_t*)act2,
                       ctx->cell_dead, ctx->cell_cnt, S, S, ctx->cells_x, cells_img);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

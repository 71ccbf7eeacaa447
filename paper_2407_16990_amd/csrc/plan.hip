// Region-aware bin packing (Alg. 1) on macroblock indexes, entirely on the GPU:
//   k_plan_label : RegionProps + Bound + Partition, one workgroup per frame (labels in LDS)
//   k_plan_rank  : Sort by importance density (rank by counting; the order is total)
//   k_plan_place : the serial first-fit over the ordered free-rectangle list, one wave,
//                  lanes test free rectangles in parallel, the list lives in LDS
//   k_plan_emit  : placement rows for boxes and macroblocks
#include "rh_internal.h"

#define NONE 0xFFFFFFFFu

__global__ void k_plan_zero(uint32_t* pcount) { if (threadIdx.x < 8) pcount[threadIdx.x] = 0; }

// One workgroup per frame.  LDS: lab[per], cminx[per], cmaxx[per], cmaxy[per] and, when it fits
// (imp_in_lds), the frame's importance values: a box leader adds up to T*T of them one after the
// other in a fixed order, which from global memory is a chain of that many load latencies.
// A region's label is the smallest in-frame index of its macroblocks.
__global__ __launch_bounds__(256) void k_plan_label(const uint8_t* __restrict__ mask,
                                                    const float* __restrict__ imp, int mbw, int mbh,
                                                    int conn, int T, int sort_policy, int imp_in_lds,
                                                    uint32_t* __restrict__ owner_id,
                                                    rh_rawbox* __restrict__ raw, uint32_t* pcount)
{
    extern __shared__ uint32_t sm[];
    const int per = mbw * mbh, tid = threadIdx.x, f = blockIdx.x;
    volatile uint32_t* lab = sm;
    uint32_t* cminx = sm + per; uint32_t* cmaxx = sm + 2 * per; uint32_t* cmaxy = sm + 3 * per;
    float* simp = (float*)(sm + 4 * per);
    __shared__ int s_changed;
    const size_t base = (size_t)f * per;
    for (int i = tid; i < per; i += 256) {
        lab[i] = mask[base + i] ? (uint32_t)i : NONE;
        cminx[i] = NONE; cmaxx[i] = 0; cmaxy[i] = 0;
        if (imp_in_lds) simp[i] = imp[base + i];
    }
    // RegionProps: iterate "take the smallest label around me, then follow it to its root"
    // until nothing changes.  Labels only decrease and always name a macroblock of the same
    // region, so the fixed point is the region's smallest index everywhere.
    for (;;) {
        __syncthreads();
        if (tid == 0) s_changed = 0;
        __syncthreads();
        int any = 0;
        for (int i = tid; i < per; i += 256) {
            uint32_t cur = lab[i];
            if (cur == NONE) continue;
            const int y = i / mbw, x = i - y * mbw;
            uint32_t m = cur;
            for (int dy = -1; dy <= 1; ++dy) {
                const int ny = y + dy;
                if (ny < 0 || ny >= mbh) continue;
                for (int dx = -1; dx <= 1; ++dx) {
                    if ((dx == 0 && dy == 0) || (conn == 4 && dx != 0 && dy != 0)) continue;
                    const int nx = x + dx;
                    if (nx < 0 || nx >= mbw) continue;
                    uint32_t ln = lab[ny * mbw + nx];
                    m = ln < m ? ln : m;
                }
            }
            for (uint32_t r = lab[m]; r < m; r = lab[m]) m = r;
            if (m < cur) { lab[i] = m; any = 1; }
        }
        if (any) s_changed = 1;
        __syncthreads();
        if (!s_changed) break;
    }
    // Bound: bounding box of every region, kept at the root's slot (min y is the root's row).
    for (int i = tid; i < per; i += 256) {
        uint32_t r = lab[i];
        if (r == NONE) continue;
        const int y = i / mbw, x = i - y * mbw;
        atomicMin(&cminx[r], (uint32_t)x); atomicMax(&cmaxx[r], (uint32_t)x); atomicMax(&cmaxy[r], (uint32_t)y);
    }
    __syncthreads();
    // Partition: the region's bounding box is cut on a T x T grid anchored at its top-left.
    // Every macroblock looks through its own cell in raster order: the first macroblock of
    // the same region there leads the box and describes it.
    for (int i = tid; i < per; i += 256) {
        uint32_t r = lab[i];
        if (r == NONE) continue;
        const int y = i / mbw, x = i - y * mbw;
        const int ry = r / mbw, minx = cminx[r], maxx = cmaxx[r], maxy = cmaxy[r];
        const int wx0 = minx + ((x - minx) / T) * T, wy0 = ry + ((y - ry) / T) * T;
        const int wx1 = min(wx0 + T - 1, maxx), wy1 = min(wy0 + T - 1, maxy);
        int leader = -1, x0 = 1 << 30, x1 = -1, y0 = 1 << 30, y1 = -1;
        float sum = 0.0f;
        for (int yy = wy0; yy <= wy1; ++yy) {
            for (int xx = wx0; xx <= wx1; ++xx) {
                const int j = yy * mbw + xx;
                if (lab[j] != r) continue;
                if (leader < 0) leader = j;
                if (leader != i) break;                      // only the leader needs the rest
                sum = __fadd_rn(sum, imp_in_lds ? simp[j] : imp[base + j]);   // fp32, ascending flat index
                x0 = min(x0, xx); x1 = max(x1, xx); y0 = min(y0, yy); y1 = max(y1, yy);
            }
            if (leader >= 0 && leader != i) break;
        }
        owner_id[base + i] = (uint32_t)(base + leader);
        if (leader == i) {
            uint32_t slot = atomicAdd(&pcount[0], 1u);
            rh_rawbox b;
            b.frame = f; b.mbx0 = x0; b.mby0 = y0; b.wmb = x1 - x0 + 1; b.hmb = y1 - y0 + 1;
            b.id = (uint32_t)(base + i); b.sum = sum;
            const int area = (x1 - x0 + 1) * (y1 - y0 + 1);
            b.key = sort_policy == RH_SORT_AREA ? (double)area : (double)sum / (double)area;
            raw[slot] = b;
        }
    }
}

// a before b in the packing order: higher key (density, or area) first, NaN last, ties by ascending id.
__device__ __forceinline__ bool box_before(double ka, uint32_t ia, double kb, uint32_t ib)
{
    const bool an = ka != ka, bn = kb != kb;
    if (an != bn) return bn;
    if (!an) { if (ka > kb) return true; if (ka < kb) return false; }
    return ia < ib;
}

// Sort by counting: the rank of a box is the number of boxes before it.
__global__ __launch_bounds__(256) void k_plan_rank(const rh_rawbox* __restrict__ raw,
                                                   const uint32_t* __restrict__ pcount,
                                                   rh_rawbox* __restrict__ sorted,
                                                   uint32_t* __restrict__ rank_of_id)
{
    __shared__ double s_key[256];
    __shared__ uint32_t s_id[256];
    const uint32_t n = pcount[0];
    if (blockIdx.x * 256u >= n) return;
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    rh_rawbox me;
    if (i < n) me = raw[i]; else { me.key = 0; me.id = 0; }
    uint32_t rank = 0;
    for (uint32_t t0 = 0; t0 < n; t0 += 256) {
        __syncthreads();
        if (t0 + threadIdx.x < n) { s_key[threadIdx.x] = raw[t0 + threadIdx.x].key; s_id[threadIdx.x] = raw[t0 + threadIdx.x].id; }
        __syncthreads();
        const uint32_t m = min(256u, n - t0);
        if (i < n)
            for (uint32_t j = 0; j < m; ++j) rank += box_before(s_key[j], s_id[j], me.key, me.id) ? 1u : 0u;
    }
    if (i < n) { sorted[rank] = me; rank_of_id[me.id] = rank; }
}

// First fit (Alg. 1 main loop) with the reading of InnerFree given in the header.
// Free rectangle j: fxy[j] = x | y<<16, fwh[j] = w | h<<16, fbin[j].
// box_pos[i] = {bin | turned<<16, bx | by<<16}; pcount[1] = n_bins, pcount[2] = overflow.
// rotate: a rectangle that cannot take the box upright may take it turned (RotatePacking).
// The loop over the boxes is serial by definition, so its cost is the latency of one step.  It
// runs in ONE wave: the 64 lanes test 64 free rectangles at a time and a ballot gives the first
// fit; LDS traffic of a single wave is executed in program order, so the list needs no barrier,
// no atomics, and every lane tracks the list length and bin count in registers.
__global__ __launch_bounds__(64) void k_plan_place(const rh_rawbox* __restrict__ sorted, uint32_t* pcount,
                                                   int halo, int S, int max_bins, int free_cap, int rotate,
                                                   uint32_t* __restrict__ box_pos)
{
    extern __shared__ uint32_t sm[];
    uint32_t* fxy = sm; uint32_t* fwh = sm + free_cap; uint32_t* fbin = sm + 2 * free_cap;
    __shared__ uint32_t s_size[256];
    const int lane = threadIdx.x;
    const uint32_t n = pcount[0];
    const int minside = RH_MB + 2 * halo;
    int nfree = 0, nbins = 0;
    uint32_t i = 0;
    bool overflow = false;
    for (; i < n && !overflow; ++i) {
        if ((i & 255u) == 0) {                                   // stage the next 256 box sizes
            for (int t = lane; t < 256; t += 64)
                if (i + t < n) s_size[t] = sorted[i + t].wmb | ((uint32_t)sorted[i + t].hmb << 16);
        }
        const uint32_t sz = s_size[i & 255u];
        int bw = RH_MB * (int)(sz & 0xFFFF) + 2 * halo, bh = RH_MB * (int)(sz >> 16) + 2 * halo;
        uint32_t at = NONE;
        for (int base = 0; base < nfree; base += 64) {           // first rectangle, in list order, that fits
            const int j = base + lane;
            bool fit = false;
            if (j < nfree) {
                const uint32_t wh = fwh[j];
                const int w = (int)(wh & 0xFFFF), h = (int)(wh >> 16);
                fit = (w >= bw && h >= bh) || (rotate && w >= bh && h >= bw);
            }
            const unsigned long long m = __ballot(fit);
            if (m) { at = (uint32_t)(base + __ffsll((long long)m) - 1); break; }
        }
        int fx, fy, fw, fh, fb, cur_n;
        if (at == NONE) {
            if (nbins >= max_bins || nfree + 2 > free_cap) { overflow = true; break; }
            at = nfree; fx = 0; fy = 0; fw = S; fh = S; fb = nbins++; cur_n = nfree + 1;
        } else {
            fx = fxy[at] & 0xFFFF; fy = fxy[at] >> 16; fw = fwh[at] & 0xFFFF; fh = fwh[at] >> 16; fb = fbin[at];
            cur_n = nfree;
            if (nfree + 1 > free_cap) { overflow = true; break; }
        }
        const bool turned = !(fw >= bw && fh >= bh);         // upright whenever that fits
        if (turned) { const int t = bw; bw = bh; bh = t; }   // occupied size
        if (lane == 0) { box_pos[2 * i] = (uint32_t)fb | (turned ? 0x10000u : 0u); box_pos[2 * i + 1] = (uint32_t)fx | ((uint32_t)fy << 16); }
        // remainder: the larger of (right strip, full height) and (bottom strip, full width),
        // plus what is left of the other
        const int ar = (fw - bw) * fh, ab = fw * (fh - bh);
        int rx = fx + bw, ry = fy, rw = fw - bw, rh, bx = fx, by = fy + bh, bwid, bhei = fh - bh;
        if (ar >= ab) { rh = fh; bwid = bw; } else { rh = bh; bwid = fw; }
        const bool keep_r = rw >= minside && rh >= minside, keep_b = bwid >= minside && bhei >= minside;
        uint32_t ixy[2], iwh[2]; int ni = 0;
        const uint32_t Rxy = rx | (ry << 16), Rwh = rw | (rh << 16), Bxy = bx | (by << 16), Bwh = bwid | (bhei << 16);
        if (keep_r && keep_b) {
            if (bwid * bhei < rw * rh) { ixy[0] = Bxy; iwh[0] = Bwh; ixy[1] = Rxy; iwh[1] = Rwh; }
            else                       { ixy[0] = Rxy; iwh[0] = Rwh; ixy[1] = Bxy; iwh[1] = Bwh; }
            ni = 2;
        } else if (keep_r) { ixy[0] = Rxy; iwh[0] = Rwh; ni = 1; }
        else if (keep_b)   { ixy[0] = Bxy; iwh[0] = Bwh; ni = 1; }
        // the survivors replace entry `at` in place: shift the tail by ni - 1
        const int delta = ni - 1, first = (int)at + 1;
        if (delta > 0) {
            for (int hi = cur_n; hi > first; hi -= 64) {         // from the top down: a chunk is read whole before it is written
                const int j = hi - 1 - lane;
                if (j >= first) { const uint32_t a = fxy[j], b = fwh[j], c = fbin[j]; fxy[j + 1] = a; fwh[j + 1] = b; fbin[j + 1] = c; }
            }
        } else if (delta < 0) {
            for (int lo = first; lo < cur_n; lo += 64) {
                const int j = lo + lane;
                if (j < cur_n) { const uint32_t a = fxy[j], b = fwh[j], c = fbin[j]; fxy[j - 1] = a; fwh[j - 1] = b; fbin[j - 1] = c; }
            }
        }
        if (lane < ni) { fxy[at + lane] = ixy[lane]; fwh[at + lane] = iwh[lane]; fbin[at + lane] = fb; }
        nfree = cur_n + delta;
    }
    // boxes that did not fit (only after an overflow)
    for (uint32_t j = i + lane; j < n; j += 64) { box_pos[2 * j] = RH_NO_BIN; box_pos[2 * j + 1] = 0; }
    if (lane == 0) { pcount[1] = nbins; pcount[2] = overflow ? 1u : 0u; }
}

__global__ __launch_bounds__(256) void k_plan_emit(const rh_rawbox* __restrict__ sorted,
                                                   const uint32_t* __restrict__ box_pos,
                                                   const uint32_t* __restrict__ pcount,
                                                   const uint32_t* __restrict__ list,
                                                   const uint32_t* __restrict__ n_sel_p,
                                                   const uint32_t* __restrict__ owner_id,
                                                   const uint32_t* __restrict__ rank_of_id, int mbw, int per,
                                                   int halo, rh_box* __restrict__ boxes,
                                                   rh_mbplace* __restrict__ places, uint32_t* __restrict__ counts)
{
    const uint32_t i = blockIdx.x * 256u + threadIdx.x;
    const uint32_t n = pcount[0], n_sel = *n_sel_p;
    if (i == 0) { counts[0] = n; counts[1] = pcount[1]; counts[2] = pcount[2]; counts[3] = n_sel; }
    if (i < n) {
        const rh_rawbox b = sorted[i];
        rh_box o;
        o.frame = b.frame; o.mbx0 = b.mbx0; o.mby0 = b.mby0; o.wmb = (uint8_t)b.wmb; o.hmb = (uint8_t)b.hmb;
        o.rot = (uint8_t)((box_pos[2 * i] >> 16) & 1u); o.pad0 = 0; o.bin = (uint16_t)(box_pos[2 * i] & 0xFFFFu);
        o.bx = (uint16_t)(box_pos[2 * i + 1] & 0xFFFF); o.by = (uint16_t)(box_pos[2 * i + 1] >> 16);
        o.pad1 = 0; o.id = b.id;
        boxes[i] = o;
    }
    if (i < n_sel) {
        const uint32_t g = list[i], rk = rank_of_id[owner_id[g]];
        const rh_rawbox b = sorted[rk];
        const uint32_t in = g % (uint32_t)per;
        const int y = in / mbw, x = in - y * mbw;
        rh_mbplace p;
        p.mb_id = g; p.box = rk; p.bin = (uint16_t)(box_pos[2 * rk] & 0xFFFFu);
        const bool placed = p.bin != RH_NO_BIN;
        const bool turned = (box_pos[2 * rk] >> 16) & 1u;
        const int dx = halo + RH_MB * (x - b.mbx0), dy = halo + RH_MB * (y - b.mby0);
        p.px = placed ? (uint16_t)((box_pos[2 * rk + 1] & 0xFFFF) + (turned ? dy : dx)) : 0;
        p.py = placed ? (uint16_t)((box_pos[2 * rk + 1] >> 16) + (turned ? dx : dy)) : 0;
        p.rot = turned ? 1 : 0;
        places[i] = p;
    }
}

rh_status rh_plan_init(rh_ctx* ctx)
{
    // Both planning kernels may need more dynamic LDS than the default limit.  The attribute belongs
    // to the kernel, not to the context: it is raised to what the largest admissible context needs
    // (rh_create bounds both sizes below 150 KB), so contexts of different sizes can coexist.
    RH_HIP(ctx, hipFuncSetAttribute((const void*)k_plan_label, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    RH_HIP(ctx, hipFuncSetAttribute((const void*)k_plan_place, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    return RH_OK;
}

rh_status rh_launch_plan(rh_ctx* ctx, int F, const float* imp, const uint8_t* mask,
                         const uint32_t* list, const uint32_t* n_sel,
                         rh_box* boxes, rh_mbplace* places, uint32_t* counts)
{
    const int per = ctx->per, total = per * F;
    uint32_t* box_pos = ctx->pcount + 8;
    rh_prof_scope ps(ctx, RH_PROF_PLAN, 5);
    hipLaunchKernelGGL(k_plan_zero, dim3(1), dim3(64), 0, ctx->stream, ctx->pcount);
    const int imp_in_lds = (size_t)per * 20 <= 150 * 1024;
    hipLaunchKernelGGL(k_plan_label, dim3(F), dim3(256), (size_t)per * (imp_in_lds ? 20 : 16), ctx->stream, mask, imp, ctx->mbw,
                       ctx->mbh, ctx->cfg.connectivity, ctx->T, ctx->cfg.sort_policy, imp_in_lds, ctx->owner_id, ctx->raw,
                       ctx->pcount);
    const int nblk = (total + 255) / 256;
    hipLaunchKernelGGL(k_plan_rank, dim3(nblk), dim3(256), 0, ctx->stream, ctx->raw, ctx->pcount, ctx->sorted,
                       ctx->rank_of_id);
    hipLaunchKernelGGL(k_plan_place, dim3(1), dim3(64), (size_t)ctx->free_cap * 12, ctx->stream, ctx->sorted,
                       ctx->pcount, ctx->cfg.halo, ctx->cfg.bin_size, ctx->cfg.max_bins, ctx->free_cap, ctx->cfg.rotate,
                       box_pos);
    hipLaunchKernelGGL(k_plan_emit, dim3(nblk), dim3(256), 0, ctx->stream, ctx->sorted, box_pos, ctx->pcount,
                       list, n_sel, ctx->owner_id, ctx->rank_of_id, ctx->mbw, per, ctx->cfg.halo, boxes, places,
                       counts);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

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

// Orders the LDS accesses of one wave: what lanes wrote before it is what any lane reads after it.
__device__ __forceinline__ void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// The packing order on integers: a larger ord_key comes first, equal keys go by ascending id.  Same
// order as box_before: doubles map to their order-preserving 64-bit image (-0 = +0), NaN to 0 (last;
// no finite key or -inf maps that low: -inf gives 0x000FFFFFFFFFFFFF).
__device__ __forceinline__ unsigned long long ord_key(double k)
{
    if (k != k) return 0ull;
    unsigned long long b = (unsigned long long)__double_as_longlong(k);
    if (b == 0x8000000000000000ull) b = 0ull;
    return (b & 0x8000000000000000ull) ? ~b : (b | 0x8000000000000000ull);
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
// runs in ONE wave.  While the free list has at most 62 entries it lives in registers, entry j in
// lane j: a ballot gives the first fit, the winner's fields are lane reads, and the entries behind
// it move up or down by one lane with a whole-wave DPP shift - no memory in the loop at all.  The
// first time the list could outgrow the wave it is written to LDS and stays there: the 64 lanes
// then test 64 rectangles at a time; the hardware executes the LDS traffic of a single wave in
// program order, and wave_sync() after every step in which lanes write what other lanes read next
// keeps the compiler from moving LDS accesses across it.  Every lane tracks the list length and
// bin count in registers.
// One wave.  sizes: box i's (wmb | hmb << 16) comes from size_of(i).  Returns through n_bins / overflow.
__device__ __forceinline__ uint32_t lane_from_below(uint32_t v)      // lane l gets lane l-1's value, lane 0 keeps its own
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x138 /* wave_shr:1 */, 0xF, 0xF, false);
}
__device__ __forceinline__ uint32_t lane_from_above(uint32_t v)      // lane l gets lane l+1's value, lane 63 keeps its own
{
    return (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x130 /* wave_shl:1 */, 0xF, 0xF, false);
}

template <typename SizeOf>
__device__ __forceinline__ void place_boxes(uint32_t n, SizeOf size_of, uint32_t* fxy, uint32_t* fwh, uint32_t* fbin,
                                            int halo, int S, int max_bins, int free_cap, int rotate,
                                            uint32_t* __restrict__ box_pos, int& n_bins_out, bool& overflow_out)
{
    const int lane = threadIdx.x & 63;
    const int minside = RH_MB + 2 * halo;
    constexpr int REG_MAX = 62;                              // a step adds at most 2 entries
    int nfree = 0, nbins = 0;
    uint32_t i = 0, szv = 0, pos0 = 0, pos1 = 0;             // lane l keeps the position of box (i & ~63) + l
    uint32_t rxy = 0, rwh = 0, rbn = 0;                      // register mode: free rectangle `lane`
    bool overflow = false;
    // Results leave in groups of 64: a global store per box would be waited for by the next box's
    // loads (stores and loads share the wave's memory counter), half a microsecond each.
    auto flush = [&](uint32_t upto) {                        // boxes [upto & ~63 ... upto) when upto is not a multiple of 64, else the last 64
        const uint32_t g0 = (upto - 1u) & ~63u;
        if (upto && g0 + lane < upto) { box_pos[2 * (g0 + lane)] = pos0; box_pos[2 * (g0 + lane) + 1] = pos1; }
    };
    // ---- register mode: the whole step is lane arithmetic and a few scalar selects ----
    for (; i < n && !overflow && nfree <= REG_MAX; ++i) {
        if ((i & 63u) == 0) {
            flush(i);
            szv = (i + lane < n) ? size_of(i + lane) : 0u;   // the next 64 box sizes, one per lane
        }
        const uint32_t sz = (uint32_t)__builtin_amdgcn_readlane((int)szv, (int)(i & 63u));
        const int bw0 = RH_MB * (int)(sz & 0xFFFF) + 2 * halo, bh0 = RH_MB * (int)(sz >> 16) + 2 * halo;
        const int w = (int)(rwh & 0xFFFF), h = (int)(rwh >> 16);
        const bool fit = lane < nfree && ((w >= bw0 && h >= bh0) || (rotate && w >= bh0 && h >= bw0));
        const unsigned long long m = __ballot(fit);
        const bool found = m != 0;
        if (found ? nfree + 1 > free_cap : (nbins >= max_bins || nfree + 2 > free_cap)) { overflow = true; break; }
        const int at = found ? __ffsll((long long)m) - 1 : nfree;              // a new bin's area goes to the end of the list
        const uint32_t lxy = (uint32_t)__builtin_amdgcn_readlane((int)rxy, at), lwh = (uint32_t)__builtin_amdgcn_readlane((int)rwh, at);
        const uint32_t lbn = (uint32_t)__builtin_amdgcn_readlane((int)rbn, at);
        const uint32_t exy = found ? lxy : 0u, ewh = found ? lwh : ((uint32_t)S | ((uint32_t)S << 16));
        const int fb = found ? (int)lbn : nbins;
        const int cur_n = found ? nfree : nfree + 1;
        nbins += found ? 0 : 1;
        const int fx = exy & 0xFFFF, fy = exy >> 16, fw = ewh & 0xFFFF, fh = ewh >> 16;
        const bool turned = !(fw >= bw0 && fh >= bh0);       // upright whenever that fits
        const int bw = turned ? bh0 : bw0, bh = turned ? bw0 : bh0;            // occupied size
        if (lane == (int)(i & 63u)) { pos0 = (uint32_t)fb | (turned ? 0x10000u : 0u); pos1 = (uint32_t)fx | ((uint32_t)fy << 16); }
        // remainder: the larger of (right strip, full height) and (bottom strip, full width),
        // plus what is left of the other
        const int rw = fw - bw, bhei = fh - bh;
        const bool right_full = rw * fh >= fw * bhei;
        const int rh = right_full ? fh : bh, bwid = right_full ? bw : fw;
        const bool keep_r = min(rw, rh) >= minside, keep_b = min(bwid, bhei) >= minside;
        const uint32_t Rxy = (uint32_t)(fx + bw) | ((uint32_t)fy << 16), Rwh = (uint32_t)rw | ((uint32_t)rh << 16);
        const uint32_t Bxy = (uint32_t)fx | ((uint32_t)(fy + bh) << 16), Bwh = (uint32_t)bwid | ((uint32_t)bhei << 16);
        const bool b_first = keep_b && (!keep_r || bwid * bhei < rw * rh);     // both kept: the smaller one first
        const uint32_t e0xy = b_first ? Bxy : Rxy, e0wh = b_first ? Bwh : Rwh, e1xy = b_first ? Rxy : Bxy, e1wh = b_first ? Rwh : Bwh;
        const int ni = (keep_r ? 1 : 0) + (keep_b ? 1 : 0);
        // the survivors replace entry `at`: the entries behind it move by ni - 1 lanes
        const uint32_t dxy = lane_from_below(rxy), dwh = lane_from_below(rwh), dbn = lane_from_below(rbn);
        const uint32_t uxy = lane_from_above(rxy), uwh = lane_from_above(rwh), ubn = lane_from_above(rbn);
        const bool down = ni == 2 && lane > at + 1, up = ni == 0 && lane >= at;
        rxy = down ? dxy : up ? uxy : rxy; rwh = down ? dwh : up ? uwh : rwh; rbn = down ? dbn : up ? ubn : rbn;
        const bool s0 = ni > 0 && lane == at, s1 = ni > 1 && lane == at + 1;
        rxy = s0 ? e0xy : s1 ? e1xy : rxy; rwh = s0 ? e0wh : s1 ? e1wh : rwh; rbn = (s0 || s1) ? (uint32_t)fb : rbn;
        nfree = cur_n + ni - 1;
    }
    // ---- the list has outgrown the wave: it moves to LDS for the rest of the boxes ----
    if (i < n && !overflow) {
        if (lane < nfree) { fxy[lane] = rxy; fwh[lane] = rwh; fbin[lane] = rbn; }
        wave_sync();
    }
    for (; i < n && !overflow; ++i) {
        if ((i & 63u) == 0) {
            flush(i);
            szv = (i + lane < n) ? size_of(i + lane) : 0u;
        }
        const uint32_t sz = (uint32_t)__builtin_amdgcn_readlane((int)szv, (int)(i & 63u));
        int bw = RH_MB * (int)(sz & 0xFFFF) + 2 * halo, bh = RH_MB * (int)(sz >> 16) + 2 * halo;
        // first rectangle, in list order, that fits: every lane reads one entry whole, the winner's
        // fields are then taken from its lane
        uint32_t at = NONE, exy = 0, ewh = 0, ebin = 0;
        for (int base = 0; base < nfree; base += 64) {
            const int j = base + lane;
            uint32_t wh = 0, xy = 0, bn = 0;
            if (j < nfree) { wh = fwh[j]; xy = fxy[j]; bn = fbin[j]; }
            const int w = (int)(wh & 0xFFFF), h = (int)(wh >> 16);
            const bool fit = j < nfree && ((w >= bw && h >= bh) || (rotate && w >= bh && h >= bw));
            const unsigned long long m = __ballot(fit);
            if (m) {
                const int l = __ffsll((long long)m) - 1;
                at = (uint32_t)(base + l);
                exy = (uint32_t)__builtin_amdgcn_readlane((int)xy, l); ewh = (uint32_t)__builtin_amdgcn_readlane((int)wh, l);
                ebin = (uint32_t)__builtin_amdgcn_readlane((int)bn, l);
                break;
            }
        }
        int fx, fy, fw, fh, fb, cur_n;
        if (at == NONE) {
            if (nbins >= max_bins || nfree + 2 > free_cap) { overflow = true; break; }
            at = nfree; fx = 0; fy = 0; fw = S; fh = S; fb = nbins++; cur_n = nfree + 1;
        } else {
            fx = exy & 0xFFFF; fy = exy >> 16; fw = ewh & 0xFFFF; fh = ewh >> 16; fb = ebin;
            cur_n = nfree;
            if (nfree + 1 > free_cap) { overflow = true; break; }
        }
        const bool turned = !(fw >= bw && fh >= bh);         // upright whenever that fits
        if (turned) { const int t = bw; bw = bh; bh = t; }   // occupied size
        if (lane == (int)(i & 63u)) { pos0 = (uint32_t)fb | (turned ? 0x10000u : 0u); pos1 = (uint32_t)fx | ((uint32_t)fy << 16); }
        const int ar = (fw - bw) * fh, ab = fw * (fh - bh);
        int rx = fx + bw, ry = fy, rw = fw - bw, rh, bx = fx, by = fy + bh, bwid, bhei = fh - bh;
        if (ar >= ab) { rh = fh; bwid = bw; } else { rh = bh; bwid = fw; }
        const bool keep_r = rw >= minside && rh >= minside, keep_b = bwid >= minside && bhei >= minside;
        uint32_t ixy[2] = {0, 0}, iwh[2] = {0, 0}; int ni = 0;
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
                uint32_t a = 0, b = 0, c = 0;
                if (j >= first) { a = fxy[j]; b = fwh[j]; c = fbin[j]; }
                wave_sync();
                if (j >= first) { fxy[j + 1] = a; fwh[j + 1] = b; fbin[j + 1] = c; }
                wave_sync();
            }
        } else if (delta < 0) {
            for (int lo = first; lo < cur_n; lo += 64) {
                const int j = lo + lane;
                uint32_t a = 0, b = 0, c = 0;
                if (j < cur_n) { a = fxy[j]; b = fwh[j]; c = fbin[j]; }
                wave_sync();
                if (j < cur_n) { fxy[j - 1] = a; fwh[j - 1] = b; fbin[j - 1] = c; }
                wave_sync();
            }
        }
        if (lane < ni) { fxy[at + lane] = ixy[lane]; fwh[at + lane] = iwh[lane]; fbin[at + lane] = fb; }
        wave_sync();
        nfree = cur_n + delta;
    }
    flush(i);                                                // i = boxes placed
    // boxes that did not fit (only after an overflow)
    for (uint32_t j = i + lane; j < n; j += 64) { box_pos[2 * j] = RH_NO_BIN; box_pos[2 * j + 1] = 0; }
    n_bins_out = nbins; overflow_out = overflow;
}

__global__ __launch_bounds__(64) void k_plan_place(const rh_rawbox* __restrict__ sorted, uint32_t* pcount,
                                                   int halo, int S, int max_bins, int free_cap, int rotate,
                                                   uint32_t* __restrict__ box_pos)
{
    extern __shared__ uint32_t sm[];
    int nbins; bool overflow;
    place_boxes(pcount[0], [&](uint32_t i) { return (uint32_t)sorted[i].wmb | ((uint32_t)sorted[i].hmb << 16); },
                sm, sm + free_cap, sm + 2 * free_cap, halo, S, max_bins, free_cap, rotate, box_pos, nbins, overflow);
    if (threadIdx.x == 0) { pcount[1] = nbins; pcount[2] = overflow ? 1u : 0u; }
}

// Placement rows of box i and of selected macroblock i (Alg. 1's output).
__device__ __forceinline__ void emit_rows(uint32_t i, uint32_t n, uint32_t n_sel, const rh_rawbox* __restrict__ sorted,
                                          const uint32_t* __restrict__ box_pos, const uint32_t* __restrict__ list,
                                          const uint32_t* __restrict__ owner_id, const uint32_t* __restrict__ rank_of_id,
                                          int mbw, int per, int halo, rh_box* __restrict__ boxes, rh_mbplace* __restrict__ places)
{
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
    emit_rows(i, n, n_sel, sorted, box_pos, list, owner_id, rank_of_id, mbw, per, halo, boxes, places);
}

// ------------------------------------------------------------------------------------------------
// The whole plan in ONE launch of one 1024-thread workgroup, for frames of at most 64 x 64
// macroblocks (1024 x 1024 pixels; the paper's streams are 640 x 360).  A plan is a few hundred
// boxes: five dependent launches cost more than the work itself.
//   A  label + bound + partition: one wave per frame (16 frames at a time), no barriers.  Lane y
//      holds row y of the frame's selection as a 64-bit mask.  A region grows from its first
//      macroblock in raster order (= its smallest index, its label): rows exchange masks with the
//      rows above and below, spread by one column (8-connectivity: the union of the three, 4: only
//      the row's own), and fill whole horizontal runs with two carry-propagating additions, until
//      nothing changes.  The region's bounding box is cut on the T x T grid; one lane per cell
//      walks the cell's rows (masks fetched from the row lanes), tightens the bounds, adds the
//      importance values in ascending index (fp32, from an LDS copy of the frame's map) and
//      writes the box and its macroblocks' owner.
//   B  rank by counting over all threads (keys in LDS for up to PF_KEYS boxes)
//   C  first fit by wave 0 (place_boxes), the free list in LDS
//   D  placement rows by all threads
#define PF_THREADS 1024
#define PF_WAVES (PF_THREADS / 64)
#define PF_KEYS 2048
#define PF_MAX_PER 2304                   // 16 waves x per x 4 B of importance <= 144 KB

typedef unsigned long long u64;

__device__ __forceinline__ u64 fill_runs(u64 n, u64 m)     // extend the bits of n (a subset of m) along the runs of ones of m
{
    const u64 up = ((m + n) ^ m) & m;                        // a carry runs from every seed to the end of its run
    const u64 rm = __brevll(m), rn = __brevll(n);
    const u64 dn = __brevll(((rm + rn) ^ rm) & rm);
    return n | up | dn;
}

struct plan_args {
    const uint8_t* mask; const float* imp; const uint32_t* list; const uint32_t* n_sel;
    int F, mbw, mbh, conn, T, sort_policy, halo, S, max_bins, free_cap, rotate;
    uint32_t* owner_id; uint32_t* rank_of_id; rh_rawbox* raw; rh_rawbox* sorted; uint32_t* box_pos;
    rh_box* boxes; rh_mbplace* places; uint32_t* counts;
};

__global__ __launch_bounds__(PF_THREADS) void k_plan_fused(plan_args a)
{
    extern __shared__ __attribute__((aligned(16))) uint32_t dyn[];
    __shared__ uint32_t s_nraw, s_nbins, s_overflow;
    __shared__ uint32_t s_sz[PF_KEYS];                       // sizes of the sorted boxes, for the first fit
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int mbw = a.mbw, mbh = a.mbh, per = mbw * mbh, T = a.T;
    if (tid == 0) s_nraw = 0;
    __syncthreads();

    // ---------------- A: regions and boxes, one wave per frame ----------------
    float* simp = (float*)dyn + (size_t)wave * per;
    for (int f = wave; f < a.F; f += PF_WAVES) {
        const size_t base = (size_t)f * per;
        for (int i = lane; i < per; i += 64) simp[i] = a.imp[base + i];
        u64 m = 0;
        for (int y = 0; y < mbh; y += 8) {                   // eight rows' loads in flight at a time
            uint8_t v8[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) v8[u] = (lane < mbw && y + u < mbh) ? a.mask[base + (size_t)(y + u) * mbw + lane] : (uint8_t)0;
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const u64 row = __ballot(v8[u] != 0);
                if (lane == y + u) m = row;
            }
        }
        wave_sync();                                         // simp is read by other lanes below
        u64 rem = m;
        for (;;) {
            const u64 rows_left = __ballot(rem != 0);
            if (!rows_left) break;
            const int ys = __ffsll((long long)rows_left) - 1;
            const u64 seed_row = __shfl(rem, ys);
            u64 comp = lane == ys ? (seed_row & (~seed_row + 1)) : 0;           // lowest set bit: the region's label
            for (;;) {                                       // RegionProps: grow until stable
                u64 up = __shfl_up(comp, 1), dn = __shfl_down(comp, 1);
                if (lane == 0) up = 0;
                if (lane == 63) dn = 0;
                u64 n;
                if (a.conn == 8) { n = comp | up | dn; n |= (n << 1) | (n >> 1); }
                else n = comp | up | dn | (comp << 1) | (comp >> 1);
                n = fill_runs((n & m) | comp, m);
                const bool changed = n != comp;
                comp = n;
                if (!__any(changed)) break;
            }
            rem &= ~comp;
            // Bound
            const u64 rows_in = __ballot(comp != 0);
            const int y0 = __ffsll((long long)rows_in) - 1, y1 = 63 - __clzll((long long)rows_in);
            u64 cols = comp;
#pragma unroll
            for (int o = 32; o > 0; o >>= 1) cols |= __shfl_xor(cols, o);
            const int x0 = __ffsll((long long)cols) - 1, x1 = 63 - __clzll((long long)cols);
            // Partition: cells of the T x T grid anchored at (x0, y0), one lane per cell
            const int ncx = (x1 - x0) / T + 1, ncy = (y1 - y0) / T + 1, cells = ncx * ncy;
            for (int c0 = 0; c0 < cells; c0 += 64) {         // uniform over the wave
                const int c = c0 + lane;
                const bool active = c < cells;
                const int cy = active ? c / ncx : 0, cx = active ? c - cy * ncx : 0;
                const int ra = y0 + cy * T, rb = min(ra + T - 1, y1), ca = x0 + cx * T, cb = min(ca + T - 1, x1);
                const u64 cmask = ((cb - ca + 1) >= 64 ? ~0ull : ((1ull << (cb - ca + 1)) - 1ull)) << ca;
                int leader = -1, bx0 = 64, bx1 = -1, by0 = 64, by1 = -1;
                float sum = 0.0f;
                const int span = min(T, y1 - y0 + 1);       // rows a cell can have: uniform
                for (int rr = 0; rr < span; ++rr) {
                    const int r = ra + rr;
                    const u64 rowbits = __shfl(comp, (active && r <= rb) ? r : 0);     // every lane takes part
                    u64 bits = (active && r <= rb) ? (rowbits & cmask) : 0;
                    if (bits) {
                        if (leader < 0) { leader = r * mbw + (__ffsll((long long)bits) - 1); by0 = r; }
                        by1 = r;
                        bx0 = min(bx0, __ffsll((long long)bits) - 1); bx1 = max(bx1, 63 - __clzll((long long)bits));
                        while (bits) {                       // ascending column = ascending flat index
                            const int x = __ffsll((long long)bits) - 1;
                            bits &= bits - 1;
                            sum = __fadd_rn(sum, simp[r * mbw + x]);
                            a.owner_id[base + r * mbw + x] = (uint32_t)(base + leader);
                        }
                    }
                }
                const bool has = leader >= 0;
                const u64 hm = __ballot(has);
                uint32_t slot0 = 0;
                if (lane == 0 && hm) slot0 = atomicAdd(&s_nraw, (uint32_t)__popcll(hm));
                slot0 = __shfl(slot0, 0);
                if (has) {
                    rh_rawbox b;
                    b.frame = f; b.mbx0 = bx0; b.mby0 = by0; b.wmb = bx1 - bx0 + 1; b.hmb = by1 - by0 + 1;
                    b.id = (uint32_t)(base + leader); b.sum = sum;
                    const int area = (bx1 - bx0 + 1) * (by1 - by0 + 1);
                    b.key = a.sort_policy == RH_SORT_AREA ? (double)area : (double)sum / (double)area;
                    a.raw[slot0 + (uint32_t)__popcll(hm & ((1ull << lane) - 1ull))] = b;
                }
            }
        }
        wave_sync();                                         // before the next frame overwrites simp
    }
    __threadfence_block();
    __syncthreads();
    const uint32_t n = s_nraw, n_sel = *a.n_sel;

    // ---------------- B: rank by counting ----------------
    u64* s_key = (u64*)dyn;
    uint32_t* s_id = (uint32_t*)(s_key + PF_KEYS);
    const bool keys_in_lds = n <= PF_KEYS;
    if (keys_in_lds)
        for (uint32_t j = tid; j < n; j += PF_THREADS) { s_key[j] = ord_key(a.raw[j].key); s_id[j] = a.raw[j].id; }
    __syncthreads();
    for (uint32_t i = tid; i < n; i += PF_THREADS) {
        const rh_rawbox me = a.raw[i];
        uint32_t rank = 0;
        if (keys_in_lds) {
            const u64 mk = ord_key(me.key);
            uint32_t j = 0;
            for (; j + 8 <= n; j += 8) {                     // eight independent LDS reads in flight
                u64 k8[8]; uint32_t d8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) { k8[u] = s_key[j + u]; d8[u] = s_id[j + u]; }
#pragma unroll
                for (int u = 0; u < 8; ++u) rank += (k8[u] > mk || (k8[u] == mk && d8[u] < me.id)) ? 1u : 0u;
            }
            for (; j < n; ++j) rank += (s_key[j] > mk || (s_key[j] == mk && s_id[j] < me.id)) ? 1u : 0u;
        } else for (uint32_t j = 0; j < n; ++j) rank += box_before(a.raw[j].key, a.raw[j].id, me.key, me.id) ? 1u : 0u;
        a.sorted[rank] = me; a.rank_of_id[me.id] = rank;
        if (rank < PF_KEYS) s_sz[rank] = (uint32_t)me.wmb | ((uint32_t)me.hmb << 16);
    }
    __threadfence_block();
    __syncthreads();                                         // keys are dead: the free list takes their place

    // ---------------- C: first fit, wave 0 ----------------
    if (wave == 0) {
        int nbins; bool overflow;
        place_boxes(n, [&](uint32_t i) { return i < PF_KEYS ? s_sz[i] : ((uint32_t)a.sorted[i].wmb | ((uint32_t)a.sorted[i].hmb << 16)); },
                    dyn, dyn + a.free_cap, dyn + 2 * a.free_cap, a.halo, a.S, a.max_bins, a.free_cap, a.rotate, a.box_pos,
                    nbins, overflow);
        if (lane == 0) { s_nbins = (uint32_t)nbins; s_overflow = overflow ? 1u : 0u; }
    }
    __threadfence_block();
    __syncthreads();

    // ---------------- D: placement rows ----------------
    if (tid == 0) { a.counts[0] = n; a.counts[1] = s_nbins; a.counts[2] = s_overflow; a.counts[3] = n_sel; }
    const uint32_t top = n > n_sel ? n : n_sel;
    for (uint32_t i = tid; i < top; i += PF_THREADS)
        emit_rows(i, n, n_sel, a.sorted, a.box_pos, a.list, a.owner_id, a.rank_of_id, mbw, per, a.halo, a.boxes, a.places);
}

rh_status rh_plan_init(rh_ctx* ctx)
{
    // The planning kernels may need more dynamic LDS than the default limit.  The attribute belongs
    // to the kernel, not to the context: it is raised to what the largest admissible context needs
    // (rh_create bounds the sizes below 150 KB), so contexts of different sizes can coexist.
    RH_HIP(ctx, hipFuncSetAttribute((const void*)k_plan_label, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    RH_HIP(ctx, hipFuncSetAttribute((const void*)k_plan_place, hipFuncAttributeMaxDynamicSharedMemorySize, 150 * 1024));
    RH_HIP(ctx, hipFuncSetAttribute((const void*)k_plan_fused, hipFuncAttributeMaxDynamicSharedMemorySize, 144 * 1024));
    return RH_OK;
}

rh_status rh_launch_plan(rh_ctx* ctx, int F, const float* imp, const uint8_t* mask,
                         const uint32_t* list, const uint32_t* n_sel,
                         rh_box* boxes, rh_mbplace* places, uint32_t* counts)
{
    const int per = ctx->per, total = per * F;
    uint32_t* box_pos = ctx->pcount + 8;
    if (ctx->mbw <= 64 && ctx->mbh <= 64 && per <= PF_MAX_PER) {
        // the usual case: everything in one launch
        size_t lds = (size_t)PF_WAVES * per * 4;
        if (lds < (size_t)PF_KEYS * 12) lds = (size_t)PF_KEYS * 12;
        if (lds < (size_t)ctx->free_cap * 12) lds = (size_t)ctx->free_cap * 12;
        plan_args a;
        a.mask = mask; a.imp = imp; a.list = list; a.n_sel = n_sel;
        a.F = F; a.mbw = ctx->mbw; a.mbh = ctx->mbh; a.conn = ctx->cfg.connectivity; a.T = ctx->T;
        a.sort_policy = ctx->cfg.sort_policy; a.halo = ctx->cfg.halo; a.S = ctx->cfg.bin_size; a.max_bins = ctx->cfg.max_bins;
        a.free_cap = ctx->free_cap; a.rotate = ctx->cfg.rotate;
        a.owner_id = ctx->owner_id; a.rank_of_id = ctx->rank_of_id; a.raw = ctx->raw; a.sorted = ctx->sorted; a.box_pos = box_pos;
        a.boxes = boxes; a.places = places; a.counts = counts;
        rh_prof_scope ps(ctx, RH_PROF_PLAN, 1);
        hipLaunchKernelGGL(k_plan_fused, dim3(1), dim3(PF_THREADS), lds, ctx->stream, a);
        RH_HIP(ctx, hipGetLastError());
        return RH_OK;
    }
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

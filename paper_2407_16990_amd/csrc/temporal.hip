// Temporal importance reuse (Sec. 3.2.2): the inverse-area operator on luma residuals, the frame
// choice by equal cuts of the cumulative change, and the copy of importance maps to the frames
// that reuse them.
//
// Phi of a frame = sum over the 8-connected blobs of changed pixels (|residual| > tau) of
// floor(2^32 / area).  Blobs are labelled in two levels, so that the residual is read once and
// everything after that touches only a small part of the pixels:
//   k_tr_reset   clears Phi and the list counters
//   k_tr_init    one workgroup per tile of 64 x 32 pixels labels the tile in LDS by union-find
//                (runs of a row start joined; rows are joined where two runs first meet) and
//                counts the pixels of every piece.  To memory go: for every piece its root
//                pixel (label = itself, area = pixel count, appended to the frame's root list)
//                and for every changed pixel on the tile's border its label = the piece's root
//                (appended to the frame's border list).  Other pixels leave no trace.
//   k_tr_merge   walks the border lists and joins the pieces that touch across tile borders
//                (lock-free union-find on the labels in memory; the trees are a few tiles deep)
//   k_tr_count   walks the root lists: a piece that is no longer a root adds its area to its root
//   k_tr_phi     walks the root lists: every remaining root is one blob and adds
//                floor(2^32 / area) to its frame's Phi
// One list and one counter per frame: a single counter for the batch would serialise the
// appends of all waves at one address.  All sums are integer, so the result does not depend on
// the order in which lanes arrive or in which the lists were filled.
#include "rh_internal.h"

struct tr_geom { int H, W; uint32_t per; };

__device__ __forceinline__ int tr_changed(const int16_t* __restrict__ res, size_t frame_base, int y, int x,
                                           int H, int W, int tau)
{
    if (y < 0 || x < 0 || x >= W || y >= H) return 0;
    const int v = res[frame_base + (size_t)y * W + x];
    return (v < 0 ? -v : v) > tau;
}

__global__ void k_tr_reset(unsigned long long* phi, int F, uint32_t* n_border, uint32_t* n_roots)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < F) { phi[i] = 0; n_border[i] = 0; n_roots[i] = 0; }
}

#define TR_ROWS 8                  // rows per wave in k_tr_init
#define TR_WAVES 4                 // waves per workgroup of k_tr_init
#define TR_TILE_H (TR_WAVES * TR_ROWS)    // a workgroup labels a tile of 64 x 32 pixels

__device__ __forceinline__ uint32_t tr_lds_find(uint32_t* lab, uint32_t x)
{
    for (;;) {                                                   // lab[x] <= x and only decreases
        const uint32_t p = __hip_atomic_load(&lab[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
        if (p == x) return x;
        x = p;
    }
}

__device__ __forceinline__ void tr_lds_union(uint32_t* lab, uint32_t a, uint32_t b)
{
    for (;;) {                                                   // as tr_union below, on the tile's labels in LDS
        a = tr_lds_find(lab, a);
        b = tr_lds_find(lab, b);
        if (a == b) return;
        if (a < b) { const uint32_t t = a; a = b; b = t; }
        const uint32_t old = atomicMin(&lab[a], b);
        if (old == a) return;
        a = old;
    }
}

// Lanes of tile row ly whose pixel can touch another tile: the top and bottom rows, the first and
// last column.  These pixels get a label in memory, because k_tr_merge may name them.
__device__ __forceinline__ uint64_t tr_edge(int ly)
{
    return (ly == 0 || ly == TR_TILE_H - 1) ? ~0ull : 0x8000000000000001ull;
}

// The border pixels from which k_tr_merge starts a join: those of the bottom row are only ever the
// other end of one.
__device__ __forceinline__ uint64_t tr_listed(int ly) { return ly == 0 ? ~0ull : 0x8000000000000001ull; }

template <bool WIDE>
__global__ __launch_bounds__(64 * TR_WAVES) void k_tr_init(const int16_t* __restrict__ res, tr_geom g, int tau,
                                                 uint32_t* __restrict__ label, uint32_t* __restrict__ area,
                                                 uint32_t* __restrict__ border, uint32_t* n_border,
                                                 uint32_t* __restrict__ roots, uint32_t* n_roots)
{
    __shared__ uint32_t s_lab[TR_TILE_H * 64];
    __shared__ uint32_t s_cnt[TR_TILE_H * 64];
    __shared__ unsigned long long s_mask[TR_TILE_H];
    __shared__ __attribute__((aligned(16))) uint32_t s_mine[4];
    __shared__ __attribute__((aligned(16))) int16_t s_res[WIDE ? TR_TILE_H * 64 : 8];
    const int lane = threadIdx.x & 63, ly0 = (threadIdx.x >> 6) * TR_ROWS;
    const int tx0 = blockIdx.x * 64, ty0 = blockIdx.y * TR_TILE_H;
    const int f = blockIdx.z, x = tx0 + lane;
    const size_t base = (size_t)f * g.per;
    const uint64_t below = (1ull << lane) - 1ull;
    int fg[TR_ROWS];
    uint64_t m[TR_ROWS];
    if constexpr (WIDE) {
        // The tile's residuals come in as 16-byte pieces (one per thread: row t/8, pixels 8*(t%8)..+7)
        // and every lane then picks its pixels out of LDS: one memory instruction per wave instead
        // of one per row.  Needs W % 8 == 0 and a 16-byte aligned tensor (pieces are then wholly
        // inside or outside a row).
        static_assert(TR_WAVES == 4, "one 16-byte piece per thread covers a 64 x 32 tile");
        const int prow = ty0 + (int)(threadIdx.x >> 3), px = tx0 + (int)(threadIdx.x & 7) * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (prow < g.H && px < g.W) v = *(const uint4*)(res + base + (size_t)prow * g.W + px);
        ((uint4*)s_res)[threadIdx.x] = v;
        __syncthreads();
#pragma unroll
        for (int j = 0; j < TR_ROWS; ++j) {
            const int r = s_res[(ly0 + j) * 64 + lane];
            fg[j] = (r < 0 ? -r : r) > tau;                      // zero-filled outside the frame
        }
    } else {
#pragma unroll
        for (int j = 0; j < TR_ROWS; ++j) fg[j] = tr_changed(res, base, ty0 + ly0 + j, x, g.H, g.W, tau);   // 0 outside the frame
    }
    uint32_t mine = 0;                                           // changed pixels of this wave's rows
#pragma unroll
    for (int j = 0; j < TR_ROWS; ++j) {
        m[j] = __ballot(fg[j]);
        mine += (uint32_t)__popcll(m[j]);
        if (lane == 0) s_mask[ly0 + j] = m[j];
        if (fg[j]) {
            const uint64_t gaps_below = ~m[j] & below;           // unchanged pixels left of this lane
            const int start = gaps_below ? 64 - __clzll((long long)gaps_below) : 0;
            s_lab[(ly0 + j) * 64 + lane] = (uint32_t)((ly0 + j) * 64 + start);   // leftmost pixel of the run
            s_cnt[(ly0 + j) * 64 + lane] = 0;
        }
    }
    if (lane == 0) s_mine[threadIdx.x >> 6] = mine;
    __syncthreads();
    {   // nothing changed in this tile (most tiles): all waves leave
        uint32_t any = 0;
#pragma unroll
        for (int i = 0; i < TR_WAVES; ++i) any |= s_mine[i];
        if (any == 0) return;
    }
    // contacts with the row above inside the tile; pixels of one run are joined already, so a
    // contact only counts where the left neighbour did not make the same one
#pragma unroll
    for (int j = 0; j < TR_ROWS; ++j) {
        const int ly = ly0 + j;
        if (ly == 0 || !fg[j]) continue;
        const uint64_t up = s_mask[ly - 1];
        const int w = lane > 0 && ((m[j] >> (lane - 1)) & 1), nn = (int)((up >> lane) & 1);
        const int nw = lane > 0 && ((up >> (lane - 1)) & 1), ne = lane < 63 && ((up >> (lane + 1)) & 1);
        const uint32_t me = (uint32_t)(ly * 64 + lane);
        if (nn) { if (!(w && nw)) tr_lds_union(s_lab, me, me - 64); }
        else {
            if (nw && !w) tr_lds_union(s_lab, me, me - 65);
            if (ne) tr_lds_union(s_lab, me, me - 63);
        }
    }
    __syncthreads();
    // pixel counts of the pieces: one LDS atomic per distinct root of a row
    uint32_t root[TR_ROWS];
    uint32_t nb = 0;                                             // border pixels of this wave's rows
#pragma unroll
    for (int j = 0; j < TR_ROWS; ++j) {
        root[j] = 0;
        if (fg[j]) root[j] = tr_lds_find(s_lab, (uint32_t)((ly0 + j) * 64 + lane));
        uint64_t pending = m[j];
        while (pending) {                                        // wave-uniform
            const int leader = __ffsll((long long)pending) - 1;
            const uint32_t r0 = (uint32_t)__shfl((int)root[j], leader);
            const uint64_t same = __ballot(fg[j] && root[j] == r0);
            if (lane == leader) atomicAdd(&s_cnt[r0], (uint32_t)__popcll(same));
            pending &= ~same;
        }
        nb += (uint32_t)__popcll(m[j] & tr_listed(ly0 + j));
    }
    __syncthreads();
    if (mine == 0) return;                                       // the same for the whole wave, and no barrier follows
    uint64_t mr[TR_ROWS];                                        // which lanes hold the root of a piece
    uint32_t nr = 0;
#pragma unroll
    for (int j = 0; j < TR_ROWS; ++j) {
        mr[j] = __ballot(fg[j] && root[j] == (uint32_t)((ly0 + j) * 64 + lane));
        nr += (uint32_t)__popcll(mr[j]);
    }
    // room in the frame's two lists: both atomics are in flight together, their latency is what
    // a workgroup of this kernel mostly waits for
    uint32_t slot_b = 0, slot_r = 0;
    if (lane == 0) {
        if (nb) slot_b = atomicAdd(&n_border[f], nb);
        if (nr) slot_r = atomicAdd(&n_roots[f], nr);
    }
    slot_b = (uint32_t)__shfl((int)slot_b, 0);
    slot_r = (uint32_t)__shfl((int)slot_r, 0);
#pragma unroll
    for (int j = 0; j < TR_ROWS; ++j) {
        const uint32_t p = (uint32_t)(base + (size_t)(ty0 + ly0 + j) * g.W + x);
        // border pixels: label = the piece's root, as a pixel index of the batch
        const uint64_t edge = tr_edge(ly0 + j), listed = tr_listed(ly0 + j), mb = m[j] & listed;
        if (fg[j] && ((edge >> lane) & 1)) {
            label[p] = (uint32_t)(base + (size_t)(ty0 + (int)(root[j] >> 6)) * g.W + tx0 + (int)(root[j] & 63));
            if ((listed >> lane) & 1) border[base + slot_b + (uint32_t)__popcll(mb & below)] = p;   // frame f's lists start at f * per
        }
        slot_b += (uint32_t)__popcll(mb);
        // roots of the pieces: label = itself, area = the piece's pixel count
        if ((mr[j] >> lane) & 1) {
            label[p] = p;
            area[p] = s_cnt[(ly0 + j) * 64 + lane];
            roots[base + slot_r + (uint32_t)__popcll(mr[j] & below)] = p;
        }
        slot_r += (uint32_t)__popcll(mr[j]);
    }
}

__device__ __forceinline__ uint32_t tr_find(uint32_t* label, uint32_t x)
{
    // Labels only ever decrease and label[x] <= x, so this walk ends at a root.  On the way every
    // visited pixel is pointed at its grandparent (still an ancestor, still smaller), which keeps
    // the chains that later walks meet short.
    for (;;) {
        const uint32_t p = __hip_atomic_load(&label[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (p == x) return x;
        const uint32_t gp = __hip_atomic_load(&label[p], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (gp == p) return p;
        atomicMin(&label[x], gp);
        x = gp;
    }
}

// Lock-free union by smaller index.  When the atomic finds that `a` was no root any more, the
// set that `a` had pointed to still has to be joined with `b`: the loop goes on with it.
__device__ __forceinline__ void tr_union(uint32_t* label, uint32_t a, uint32_t b)
{
    for (;;) {
        a = tr_find(label, a);
        b = tr_find(label, b);
        if (a == b) return;
        if (a < b) { const uint32_t t = a; a = b; b = t; }
        const uint32_t old = atomicMin(&label[a], b);
        if (old == a) return;
        a = old;
    }
}

// The three list kernels run a fixed grid (x: workgroups of one frame, y: frame); every thread
// strides over its frame's list.
__global__ __launch_bounds__(256) void k_tr_merge(const int16_t* __restrict__ res, tr_geom g, int tau,
                                                  uint32_t* label, const uint32_t* __restrict__ border,
                                                  const uint32_t* __restrict__ n_border)
{
    const uint32_t f = blockIdx.y, n = n_border[f], stride = gridDim.x * 256;
    border += (size_t)f * g.per;
    // two work items per listed pixel (0: the join to the left, 1: the joins upwards), so that no
    // thread has more than two joins - each a chain of dependent memory round trips - in a row
    for (uint32_t i2 = blockIdx.x * 256 + threadIdx.x; i2 < 2 * n; i2 += stride) {
        const uint32_t p = border[i2 >> 1];
        const uint32_t r = p - f * g.per;
        const int y = (int)(r / (uint32_t)g.W), x = (int)(r - (uint32_t)y * (uint32_t)g.W);
        const size_t base = (size_t)f * g.per;
        const int lx = x & 63, ly = y % TR_TILE_H;
        // The rule k_tr_init uses inside a tile (runs are joined, so a contact with the row above
        // counts only where the left neighbour did not make the same one), applied to the
        // contacts that cross a tile border; the neighbour then lies on its own tile's border
        // and has a label.
        if ((i2 & 1) == 0) {
            if (lx == 0 && tr_changed(res, base, y, x - 1, g.H, g.W, tau)) tr_union(label, p, p - 1);
            continue;
        }
        const int w = tr_changed(res, base, y, x - 1, g.H, g.W, tau), nn = tr_changed(res, base, y - 1, x, g.H, g.W, tau);
        const int nw = tr_changed(res, base, y - 1, x - 1, g.H, g.W, tau), ne = tr_changed(res, base, y - 1, x + 1, g.H, g.W, tau);
        if (nn) { if (ly == 0 && !(w && nw)) tr_union(label, p, p - (uint32_t)g.W); }
        else {
            if (nw && !w && (ly == 0 || lx == 0)) tr_union(label, p, p - (uint32_t)g.W - 1);
            if (ne && (ly == 0 || lx == 63)) tr_union(label, p, p - (uint32_t)g.W + 1);
        }
    }
}

__global__ __launch_bounds__(256) void k_tr_count(tr_geom g, uint32_t* label, uint32_t* area, const uint32_t* __restrict__ roots,
                                                  const uint32_t* __restrict__ n_roots)
{
    const uint32_t n = n_roots[blockIdx.y], stride = gridDim.x * 256;
    roots += (size_t)blockIdx.y * g.per;
    for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const uint32_t p = roots[i];
        const uint32_t r = tr_find(label, p);
        // only final roots are added to, and a final root adds nothing: area[p] is not written here
        if (r != p) atomicAdd(&area[r], area[p]);
    }
}

__global__ __launch_bounds__(256) void k_tr_phi(tr_geom g, const uint32_t* __restrict__ label,
                                                const uint32_t* __restrict__ area, uint32_t min_area,
                                                const uint32_t* __restrict__ roots, const uint32_t* __restrict__ n_roots,
                                                unsigned long long* phi)
{
    const uint32_t n = n_roots[blockIdx.y], stride = gridDim.x * 256;
    roots += (size_t)blockIdx.y * g.per;
    for (uint32_t i = blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
        const uint32_t p = roots[i];
        if (label[p] != p) continue;                             // what is still a root is one blob
        const uint32_t a = area[p];
        if (a >= min_area) atomicAdd(&phi[blockIdx.y], (1ull << 32) / a);
    }
}

rh_status rh_launch_temporal_phi(rh_ctx* ctx, const int16_t* res, int F, int tau, int min_area, uint64_t* phi)
{
    const int H = ctx->cfg.frame_h, W = ctx->cfg.frame_w;
    const size_t px = (size_t)F * H * W;
    if (px >= 0x7FFFFFFFull) RH_FAIL(ctx, RH_E_SHAPE, "rh_temporal_phi: %zu pixels exceed the 32-bit label range", px);
    if (F > 65535) RH_FAIL(ctx, RH_E_CAPACITY, "rh_temporal_phi: F=%d exceeds 65535 frames per call", F);
    rh_status st = rh_ensure_workspace(ctx, px * 16 + (size_t)F * 8);
    if (st != RH_OK) return st;
    uint32_t* label = (uint32_t*)ctx->act;
    uint32_t* area = label + px;
    uint32_t* border = area + px;
    uint32_t* roots = border + px;
    uint32_t* n_border = roots + px;
    uint32_t* n_roots = n_border + F;
    tr_geom g{H, W, (uint32_t)((size_t)H * W)};
    const dim3 grid((W + 63) / 64, (H + TR_TILE_H - 1) / TR_TILE_H, F), block(256);
    rh_prof_scope ps(ctx, RH_PROF_TEMPORAL, 5);
    hipLaunchKernelGGL(k_tr_reset, dim3((F + 255) / 256), block, 0, ctx->stream, (unsigned long long*)phi, F, n_border, n_roots);
    if (TR_WAVES == 4 && W % 8 == 0 && ((uintptr_t)res & 15) == 0)
        hipLaunchKernelGGL(k_tr_init<true>, grid, dim3(64 * TR_WAVES), 0, ctx->stream, res, g, tau, label, area, border, n_border, roots, n_roots);
    else
        hipLaunchKernelGGL(k_tr_init<false>, grid, dim3(64 * TR_WAVES), 0, ctx->stream, res, g, tau, label, area, border, n_border, roots, n_roots);
    hipLaunchKernelGGL(k_tr_merge, dim3(16, F), block, 0, ctx->stream, res, g, tau, label, (const uint32_t*)border,
                       (const uint32_t*)n_border);
    hipLaunchKernelGGL(k_tr_count, dim3(8, F), block, 0, ctx->stream, g, label, area, (const uint32_t*)roots,
                       (const uint32_t*)n_roots);
    hipLaunchKernelGGL(k_tr_phi, dim3(8, F), block, 0, ctx->stream, g, (const uint32_t*)label, (const uint32_t*)area,
                       (uint32_t)min_area, (const uint32_t*)roots, (const uint32_t*)n_roots, (unsigned long long*)phi);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

// ---------------------------------------------------------------------------------------------
// Frame choice.  Everything is decided by exact comparisons of products of 64-bit integers.

struct u128 { uint64_t hi, lo; };
__device__ __forceinline__ u128 mul64(uint64_t a, uint64_t b) { return u128{__umul64hi(a, b), a * b}; }
__device__ __forceinline__ bool le128(u128 a, u128 b) { return a.hi < b.hi || (a.hi == b.hi && a.lo <= b.lo); }
__device__ __forceinline__ bool lt128(u128 a, u128 b) { return a.hi < b.hi || (a.hi == b.hi && a.lo < b.lo); }
__device__ __forceinline__ u128 sub128(u128 a, u128 b) { return u128{a.hi - b.hi - (a.lo < b.lo ? 1u : 0u), a.lo - b.lo}; }
__device__ __forceinline__ u128 absdiff128(u128 a, u128 b) { return le128(b, a) ? sub128(a, b) : sub128(b, a); }

#define TR_MAX_CHUNK 2048      // frames of one stream's chunk
#define TR_MAX_STREAMS 1024

struct tr_off_chunk { int32_t first, n; int32_t v[512]; };

__global__ void k_tr_upload(tr_off_chunk c, int32_t* off)
{
    for (int i = threadIdx.x; i < c.n; i += blockDim.x) off[c.first + i] = c.v[i];
}

// One workgroup per stream: S_i = |Phi_{i+1} - Phi_i|, A_f = S_0 + ... + S_{f-1}, total = A_{n-1}.
__global__ __launch_bounds__(256) void k_tr_prefix(const unsigned long long* __restrict__ phi, const int32_t* __restrict__ off,
                                                   unsigned long long* __restrict__ A, unsigned long long* __restrict__ total,
                                                   uint32_t* n_selected)
{
    __shared__ unsigned long long s_sum[256];
    const int s = blockIdx.x, t = threadIdx.x, b = off[s], n = off[s + 1] - b;
    if (s == 0 && t == 0) *n_selected = 0;
    unsigned long long S[8], mine = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int i = t * 8 + j;
        S[j] = 0;
        if (i + 1 < n) {
            const unsigned long long u = phi[b + i], v = phi[b + i + 1];
            S[j] = u > v ? u - v : v - u;
        }
        mine += S[j];
    }
    s_sum[t] = mine;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {                          // inclusive scan of the per-thread sums
        const unsigned long long add = t >= o ? s_sum[t - o] : 0;
        __syncthreads();
        s_sum[t] += add;
        __syncthreads();
    }
    unsigned long long run = s_sum[t] - mine;                    // sum of everything before this thread
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        const int i = t * 8 + j;
        if (i < n) A[b + i] = run;
        run += S[j];
    }
    if (t == 255) total[s] = s_sum[255];
}

// One workgroup per stream: its share N of the budget, then the interval of every frame, then the
// frame nearest the midpoint in every interval.
__global__ __launch_bounds__(256) void k_tr_choose(const unsigned long long* __restrict__ A, const unsigned long long* __restrict__ total,
                                                   const int32_t* __restrict__ off, int n_streams, int n_total,
                                                   uint32_t* __restrict__ alloc, uint8_t* __restrict__ selected,
                                                   uint32_t* __restrict__ reuse_from, uint32_t* n_selected)
{
    __shared__ unsigned long long s_red[256];
    __shared__ uint32_t s_cell[TR_MAX_CHUNK];
    __shared__ uint32_t s_dhi[TR_MAX_CHUNK];
    __shared__ unsigned long long s_dlo[TR_MAX_CHUNK];
    __shared__ uint32_t s_picked;
    const int s = blockIdx.x, t = threadIdx.x;
    const uint64_t rest = (uint64_t)(n_total - n_streams);

    // ---- share of the budget: 1 + floor(rest * T_s / whole) (+ 1 for the largest remainders)
    unsigned long long part = 0;
    for (int i = t; i < n_streams; i += 256) part += total[i];
    s_red[t] = part;
    if (t == 0) s_picked = 0;
    __syncthreads();
    for (int o = 128; o; o >>= 1) { if (t < o) s_red[t] += s_red[t + o]; __syncthreads(); }
    const uint64_t whole = s_red[0];
    __syncthreads();
    uint32_t N;
    if (whole == 0) {
        N = 1u + (uint32_t)(rest / (uint64_t)n_streams) + ((uint64_t)s < rest % (uint64_t)n_streams ? 1u : 0u);
    } else {
        // quotient and remainder of rest * T / whole without a 128-bit division: the quotient is
        // at most `rest`, found by bisection on q * whole <= rest * T
        auto share = [&](uint64_t T, uint64_t& rem) -> uint32_t {
            const u128 num = mul64(rest, T);
            uint64_t lo = 0, hi = rest;                          // invariant: lo * whole <= num
            while (lo < hi) {
                const uint64_t mid = lo + (hi - lo + 1) / 2;
                if (le128(mul64(mid, whole), num)) lo = mid; else hi = mid - 1;
            }
            rem = sub128(num, mul64(lo, whole)).lo;
            return (uint32_t)lo;
        };
        uint64_t my_rem;
        const uint32_t my_q = share(total[s], my_rem);
        unsigned long long qsum = 0, ahead = 0;                  // streams ranked before this one by remainder
        for (int i = t; i < n_streams; i += 256) {
            uint64_t r;
            qsum += share(total[i], r);
            if (r > my_rem || (r == my_rem && i < s)) ++ahead;
        }
        s_red[t] = qsum;
        __syncthreads();
        for (int o = 128; o; o >>= 1) { if (t < o) s_red[t] += s_red[t + o]; __syncthreads(); }
        const uint64_t left = rest - s_red[0];
        __syncthreads();
        s_red[t] = ahead;
        __syncthreads();
        for (int o = 128; o; o >>= 1) { if (t < o) s_red[t] += s_red[t + o]; __syncthreads(); }
        N = 1u + my_q + (s_red[0] < left ? 1u : 0u);
        __syncthreads();
    }
    if (t == 0) alloc[s] = N;

    // ---- interval of every frame and its distance from the interval's midpoint, scaled by 2*N*T
    const int b = off[s], n = off[s + 1] - b;
    const uint64_t T = total[s];
    for (int f = t; f < n; f += 256) {
        const uint64_t a = A[b + f];
        uint32_t cell = 0;
        if (T != 0) {
            const u128 na = mul64((uint64_t)N, a);
            uint32_t lo = 0, hi = N - 1;                         // largest j with j * T <= N * a
            while (lo < hi) {
                const uint32_t mid = lo + (hi - lo + 1) / 2;
                if (le128(mul64((uint64_t)mid, T), na)) lo = mid; else hi = mid - 1;
            }
            cell = lo;
        }
        const u128 d = absdiff128(mul64(2ull * N, a), mul64(2ull * cell + 1ull, T));
        s_cell[f] = cell; s_dhi[f] = (uint32_t)d.hi; s_dlo[f] = d.lo;
    }
    __syncthreads();
    // ---- the first frame of every interval walks its interval (intervals are runs of frames)
    for (int f = t; f < n; f += 256) {
        if (f > 0 && s_cell[f - 1] == s_cell[f]) continue;
        int best = f, e = f + 1;
        for (; e < n && s_cell[e] == s_cell[f]; ++e)
            if (lt128(u128{s_dhi[e], s_dlo[e]}, u128{s_dhi[best], s_dlo[best]})) best = e;
        for (int q = f; q < e; ++q) { reuse_from[b + q] = (uint32_t)(b + best); selected[b + q] = q == best; }
        atomicAdd(&s_picked, 1u);
    }
    __syncthreads();
    if (t == 0) atomicAdd(n_selected, s_picked);
}

rh_status rh_launch_temporal_select(rh_ctx* ctx, const uint64_t* phi, const int32_t* stream_off, int n_streams,
                                    int n_total, uint32_t* alloc, uint8_t* selected, uint32_t* reuse_from,
                                    uint32_t* n_selected)
{
    for (int s0 = 0; s0 <= n_streams; s0 += 512) {
        tr_off_chunk c;
        c.first = s0; c.n = (n_streams + 1 - s0) < 512 ? (n_streams + 1 - s0) : 512;
        for (int i = 0; i < c.n; ++i) c.v[i] = stream_off[s0 + i];
        hipLaunchKernelGGL(k_tr_upload, dim3(1), dim3(256), 0, ctx->stream, c, ctx->tr_off);
    }
    rh_prof_scope ps(ctx, RH_PROF_TEMPORAL, 2);
    hipLaunchKernelGGL(k_tr_prefix, dim3(n_streams), dim3(256), 0, ctx->stream, (const unsigned long long*)phi,
                       (const int32_t*)ctx->tr_off, (unsigned long long*)ctx->tr_A, (unsigned long long*)ctx->tr_T, n_selected);
    hipLaunchKernelGGL(k_tr_choose, dim3(n_streams), dim3(256), 0, ctx->stream, (const unsigned long long*)ctx->tr_A,
                       (const unsigned long long*)ctx->tr_T, (const int32_t*)ctx->tr_off, n_streams, n_total, alloc,
                       selected, reuse_from, n_selected);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

// Frames that are not predicted take the map of the frame they reuse.
__global__ __launch_bounds__(256) void k_tr_spread(float* imp, int F, int per, const uint8_t* __restrict__ selected,
                                                   const uint32_t* __restrict__ reuse_from)
{
    const int f = blockIdx.y;
    if (selected[f]) return;
    const uint32_t r = reuse_from[f];
    if (r >= (uint32_t)F || !selected[r]) return;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i < per) imp[(size_t)f * per + i] = imp[(size_t)r * per + i];
}

rh_status rh_launch_temporal_spread(rh_ctx* ctx, float* imp, int F, const uint8_t* selected, const uint32_t* reuse_from)
{
    rh_prof_scope ps(ctx, RH_PROF_TEMPORAL, 1);
    hipLaunchKernelGGL(k_tr_spread, dim3((ctx->per + 255) / 256, F), dim3(256), 0, ctx->stream, imp, F, ctx->per,
                       selected, reuse_from);
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

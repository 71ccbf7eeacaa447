// Temporal importance reuse (Sec. 3.2.2): the inverse-area operator on luma residuals, the frame
// choice by equal cuts of the cumulative change, and the copy of importance maps to the frames
// that reuse them.
//
// Phi of a frame = sum over the 8-connected blobs of changed pixels (|residual| > tau) of
// floor(2^32 / area): blob labelling by union-find on a label array in the workspace.
//   k_tr_init    one wave per 64-pixel row segment: a changed pixel starts with the index of the
//                leftmost pixel of its horizontal run inside the segment as its label
//   k_tr_merge   joins runs across segment borders and with the row above, only where two runs
//                first meet (the other contacts of the same two runs are implied by these)
//   k_tr_count   every changed pixel finds its root; one atomic add per distinct root in a wave
//   k_tr_phi     roots add floor(2^32 / area) to their frame's Phi (a wave-level sum, then one
//                64-bit atomic per wave)
// All sums are integer, so the result does not depend on the order in which lanes arrive.
#include "rh_internal.h"

#define TR_NONE 0xFFFFFFFFu

struct tr_geom { int H, W, tiles_x; uint32_t per; };

__device__ __forceinline__ int tr_changed(const int16_t* __restrict__ res, size_t frame_base, int y, int x,
                                           int H, int W, int tau)
{
    if (y < 0 || x < 0 || x >= W || y >= H) return 0;
    const int v = res[frame_base + (size_t)y * W + x];
    return (v < 0 ? -v : v) > tau;
}

__global__ __launch_bounds__(256) void k_tr_init(const int16_t* __restrict__ res, tr_geom g, int tau,
                                                 uint32_t* __restrict__ label, uint32_t* __restrict__ area,
                                                 unsigned long long* __restrict__ phi)
{
    const int lane = threadIdx.x & 63, row = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int f = blockIdx.z, x = blockIdx.x * 64 + lane;
    if (blockIdx.x == 0 && blockIdx.y == 0 && threadIdx.x == 0) phi[f] = 0;
    if (row >= g.H) return;                                      // whole waves leave together
    const size_t base = (size_t)f * g.per;
    const int fg = tr_changed(res, base, row, x, g.H, g.W, tau);
    const uint64_t m = __ballot(fg);
    if (x >= g.W) return;
    const uint32_t p = (uint32_t)(base + (size_t)row * g.W + x);
    uint32_t l = TR_NONE;
    if (fg) {
        const uint64_t gaps_below = ~m & ((1ull << lane) - 1ull);           // unchanged pixels left of this lane
        const int start = gaps_below ? 64 - __clzll((long long)gaps_below) : 0;
        l = p - (uint32_t)(lane - start);
    }
    label[p] = l;
    area[p] = 0;
}

__device__ __forceinline__ uint32_t tr_find(uint32_t* label, uint32_t x)
{
    // labels only ever decrease and label[x] <= x, so this walk ends at a root
    for (;;) {
        const uint32_t p = __hip_atomic_load(&label[x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        if (p == x) return x;
        x = p;
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

__global__ __launch_bounds__(256) void k_tr_merge(const int16_t* __restrict__ res, tr_geom g, int tau,
                                                  uint32_t* label)
{
    const int lane = threadIdx.x & 63, y = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int f = blockIdx.z, x = blockIdx.x * 64 + lane;
    if (y >= g.H || x >= g.W) return;
    const size_t base = (size_t)f * g.per;
    if (!tr_changed(res, base, y, x, g.H, g.W, tau)) return;
    const uint32_t p = (uint32_t)(base + (size_t)y * g.W + x);
    const int w = tr_changed(res, base, y, x - 1, g.H, g.W, tau);
    const int n = tr_changed(res, base, y - 1, x, g.H, g.W, tau);
    const int nw = tr_changed(res, base, y - 1, x - 1, g.H, g.W, tau);
    const int ne = tr_changed(res, base, y - 1, x + 1, g.H, g.W, tau);
    // a run that goes on from the previous 64-pixel segment
    if (w && lane == 0) tr_union(label, p, p - 1);
    // the row above: pixels of one run are joined already, so a contact only counts where the
    // left neighbour did not make the same one
    if (n) { if (!(w && nw)) tr_union(label, p, p - (uint32_t)g.W); }
    else {
        if (nw && !w) tr_union(label, p, p - (uint32_t)g.W - 1);
        if (ne) tr_union(label, p, p - (uint32_t)g.W + 1);
    }
}

__global__ __launch_bounds__(256) void k_tr_count(tr_geom g, uint32_t* label, uint32_t* area)
{
    const int lane = threadIdx.x & 63, y = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int f = blockIdx.z, x = blockIdx.x * 64 + lane;
    if (y >= g.H) return;
    uint32_t root = TR_NONE;
    int fg = 0;
    if (x < g.W) {
        const uint32_t p = (uint32_t)((size_t)f * g.per + (size_t)y * g.W + x);
        if (label[p] != TR_NONE) { fg = 1; root = tr_find(label, p); }
    }
    uint64_t pending = __ballot(fg);
    while (pending) {                                            // one round per distinct root of the wave
        const int leader = __ffsll((long long)pending) - 1;
        const uint32_t r0 = (uint32_t)__shfl((int)root, leader);
        const uint64_t same = __ballot(fg && root == r0);
        if (lane == leader) atomicAdd(&area[r0], (uint32_t)__popcll(same));
        pending &= ~same;
    }
}

__global__ __launch_bounds__(256) void k_tr_phi(tr_geom g, const uint32_t* __restrict__ label,
                                                const uint32_t* __restrict__ area, uint32_t min_area,
                                                unsigned long long* phi)
{
    const int lane = threadIdx.x & 63, y = blockIdx.y * 4 + (threadIdx.x >> 6);
    const int f = blockIdx.z, x = blockIdx.x * 64 + lane;
    if (y >= g.H) return;
    unsigned long long c = 0;
    if (x < g.W) {
        const uint32_t p = (uint32_t)((size_t)f * g.per + (size_t)y * g.W + x);
        if (label[p] == p) {
            const uint32_t a = area[p];
            if (a >= min_area) c = (1ull << 32) / a;
        }
    }
    if (__ballot(c != 0) == 0) return;
    for (int o = 32; o; o >>= 1) {
        const uint32_t lo = (uint32_t)__shfl_down((int)(uint32_t)c, o), hi = (uint32_t)__shfl_down((int)(uint32_t)(c >> 32), o);
        c += ((unsigned long long)hi << 32) | lo;
    }
    if (lane == 0) atomicAdd(&phi[f], c);
}

rh_status rh_launch_temporal_phi(rh_ctx* ctx, const int16_t* res, int F, int tau, int min_area, uint64_t* phi)
{
    const int H = ctx->cfg.frame_h, W = ctx->cfg.frame_w;
    const size_t px = (size_t)F * H * W;
    if (px >= 0x7FFFFFFFull) RH_FAIL(ctx, RH_E_SHAPE, "rh_temporal_phi: %zu pixels exceed the 32-bit label range", px);
    rh_status st = rh_ensure_workspace(ctx, px * 8);
    if (st != RH_OK) return st;
    uint32_t* label = (uint32_t*)ctx->act;
    uint32_t* area = label + px;
    tr_geom g{H, W, (W + 63) / 64, (uint32_t)((size_t)H * W)};
    const dim3 grid(g.tiles_x, (H + 3) / 4, F), block(256);
    rh_prof_scope ps(ctx, RH_PROF_TEMPORAL, 4);
    hipLaunchKernelGGL(k_tr_init, grid, block, 0, ctx->stream, res, g, tau, label, area, (unsigned long long*)phi);
    hipLaunchKernelGGL(k_tr_merge, grid, block, 0, ctx->stream, res, g, tau, label);
    hipLaunchKernelGGL(k_tr_count, grid, block, 0, ctx->stream, g, label, area);
    hipLaunchKernelGGL(k_tr_phi, grid, block, 0, ctx->stream, g, (const uint32_t*)label, (const uint32_t*)area,
                       (uint32_t)min_area, (unsigned long long*)phi);
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

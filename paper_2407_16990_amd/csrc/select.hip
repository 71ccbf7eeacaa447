// Cross-stream macroblock selection (Sec. 3.3.1): the top-k of each segment's importance
// queue, or a threshold, as an exact k-th-key radix select plus an ordered ballot/prefix-sum
// compaction.  No sort of the queue is materialised: a macroblock is selected iff its key is
// above the k-th key, or equals it and is among the first `budget` such macroblocks in
// ascending flat index.
#include <string.h>

#include "rh_internal.h"

// Order-preserving image of an fp32 importance: larger key = more important.
// -0 is treated as +0 and every NaN maps to 0, below all numbers (-inf maps to 0x007FFFFF).
__device__ __forceinline__ uint32_t imp_key(float v)
{
    uint32_t b = __float_as_uint(v);
    if ((b & 0x7FFFFFFFu) > 0x7F800000u) return 0u;
    if (b == 0x80000000u) b = 0u;
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}

// Kernel 1: one workgroup per segment.  Finds the segment's threshold key T and tie budget,
// then the number of selected macroblocks and admitted ties of each of its frames.
// seg_par[seg] = {g_begin, g_end, k, thr bits}.
// A queue of up to KREG * 1024 keys (a 30-frame chunk of 480x272 streams is 15k) is read from
// global memory once and kept in registers over the four radix passes.
#define KREG 16
#define FCHUNK 1024          // frames whose counts are held in LDS at a time

__device__ __forceinline__ void hist_add(uint32_t* hist, bool todo, uint32_t bin, bool aggregate)
{
    if (!aggregate) { if (todo) atomicAdd(&hist[bin], 1u); return; }
    // the top byte (sign and exponent) can put most keys of a wave into a few bins, which would
    // serialise their atomics: the lanes that share the bin of the first pending lane are counted
    // with one ballot and added by one lane, twice; what is left after that is spread out
    unsigned long long act = __ballot(todo);
#pragma unroll
    for (int round = 0; round < 2; ++round) {
        if (!act) break;
        const int first = __ffsll((long long)act) - 1;
        const uint32_t b = (uint32_t)__builtin_amdgcn_readlane((int)bin, first);
        const unsigned long long same = __ballot(todo && bin == b);
        if ((int)(threadIdx.x & 63) == first) atomicAdd(&hist[b], (uint32_t)__popcll(same));
        act &= ~same;
        todo = todo && bin != b;
    }
    if (todo) atomicAdd(&hist[bin], 1u);
}

__global__ __launch_bounds__(1024) void k_select_kth(const float* __restrict__ imp,
                                                     const uint32_t* __restrict__ seg_par, int mode,
                                                     int per, uint32_t* __restrict__ seg_T,
                                                     uint32_t* __restrict__ frame_nsel,
                                                     uint32_t* __restrict__ frame_ties)
{
    __shared__ uint32_t hist[256];
    __shared__ uint32_t s_wtot[4];
    __shared__ uint32_t s_prefix, s_remaining;
    __shared__ uint32_t s_gt[FCHUNK], s_eq[FCHUNK], s_scan[2][FCHUNK];
    const int tid = threadIdx.x, seg = blockIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    const uint32_t g0 = seg_par[4 * seg], g1 = seg_par[4 * seg + 1];
    const uint32_t n = g1 - g0;
    const uint32_t f0 = g0 / per, f1 = g1 / per;
    uint32_t k = seg_par[4 * seg + 2];
    // a queue that fits is read once and stays in registers for the radix passes and the counts
    const bool in_regs = n <= KREG * 1024u && f1 - f0 <= FCHUNK;
    uint32_t keys[KREG];
    if (in_regs) {
#pragma unroll
        for (int j = 0; j < KREG; ++j) {
            const uint32_t i = (uint32_t)j * 1024u + tid;
            keys[j] = i < n ? imp_key(imp[g0 + i]) : 0u;
        }
    }
    uint32_t T, budget;
    if (mode == RH_THRESHOLD) {
        float thr = __uint_as_float(seg_par[4 * seg + 3]);
        if (thr != thr) { T = 0xFFFFFFFFu; budget = 0u; }       // NaN threshold selects nothing
        else { T = imp_key(thr); budget = 0xFFFFFFFFu; }         // every key == T is taken
    } else {
        if (k > n) k = n;
        if (k == 0) { T = 0xFFFFFFFFu; budget = 0u; }            // no key reaches 0xFFFFFFFF
        else {
            uint32_t prefix = 0, remaining = k;
            for (int pass = 3; pass >= 0; --pass) {
                const int shift = pass * 8;
                const uint32_t hi_mask = (pass == 3) ? 0u : (0xFFFFFFFFu << (shift + 8));
                if (tid < 256) hist[tid] = 0;
                __syncthreads();
                if (in_regs) {
#pragma unroll
                    for (int j = 0; j < KREG; ++j) {
                        const uint32_t i = (uint32_t)j * 1024u + tid;
                        if ((uint32_t)j * 1024u < n)                 // uniform over the workgroup
                            hist_add(hist, i < n && (keys[j] & hi_mask) == prefix, (keys[j] >> shift) & 255u, pass == 3);
                    }
                } else {
                    for (uint32_t i0 = 0; i0 < n; i0 += 1024) {
                        const uint32_t i = i0 + tid;
                        const uint32_t key = i < n ? imp_key(imp[g0 + i]) : 0u;
                        hist_add(hist, i < n && (key & hi_mask) == prefix, (key >> shift) & 255u, pass == 3);
                    }
                }
                __syncthreads();
                // bin t holds the k-th key iff  above(t) < remaining <= above(t) + hist[t],  above(t) = sum of
                // the bins over t: a suffix scan by shuffles inside each of the 4 waves that hold the bins
                uint32_t h = 0, suf = 0;
                if (tid < 256) {
                    h = hist[tid]; suf = h;
#pragma unroll
                    for (int o = 1; o < 64; o <<= 1) { const uint32_t t = __shfl_down(suf, o); if (lane + o < 64) suf += t; }
                    if (lane == 0) s_wtot[wave] = suf;
                }
                __syncthreads();
                if (tid < 256) {
                    uint32_t above = suf - h;
                    for (int w = wave + 1; w < 4; ++w) above += s_wtot[w];
                    if (above < remaining && remaining <= above + h) { s_prefix = prefix | ((uint32_t)tid << shift); s_remaining = remaining - above; }
                }
                __syncthreads();
                prefix = s_prefix; remaining = s_remaining;
            }
            T = prefix; budget = remaining;
        }
    }
    if (tid == 0) seg_T[seg] = T;
    // per-frame counts of keys above T (gt) and equal to T (eq); the ties are then dealt to the
    // frames in ascending order: a frame may take  min(eq, budget - ties of the frames before it)
    uint32_t left = budget;                                    // uniform over the workgroup
    for (uint32_t c0 = f0; c0 < f1; c0 += FCHUNK) {
        const uint32_t nf = (f1 - c0) < FCHUNK ? (f1 - c0) : FCHUNK;
        if (in_regs) {                                         // one chunk: counts straight from the registers
            if ((uint32_t)tid < nf) { s_gt[tid] = 0; s_eq[tid] = 0; }
            __syncthreads();
#pragma unroll
            for (int j = 0; j < KREG; ++j) {
                if ((uint32_t)j * 1024u >= n) continue;            // uniform over the workgroup
                const uint32_t i = (uint32_t)j * 1024u + tid;
                const bool gt = i < n && keys[j] > T, eq = i < n && keys[j] == T;
                const uint32_t fr = i / (uint32_t)per;             // frame within the segment
                unsigned long long act = __ballot(gt || eq);
                while (act) {                                      // one round per frame present in the wave
                    const int first = __ffsll((long long)act) - 1;
                    const uint32_t fs = (uint32_t)__builtin_amdgcn_readlane((int)fr, first);
                    const unsigned long long mg = __ballot(gt && fr == fs), me = __ballot(eq && fr == fs);
                    const uint32_t ng = (uint32_t)__popcll(mg), ne = (uint32_t)__popcll(me);
                    if (lane == first) { if (ng) atomicAdd(&s_gt[fs], ng); if (ne) atomicAdd(&s_eq[fs], ne); }
                    act &= ~(mg | me);
                }
            }
        } else {                                               // one wave per frame, from global memory
            for (uint32_t j = wave; j < nf; j += 16) {
                const size_t fb = (size_t)(c0 + j) * per;
                uint32_t gt = 0, eq = 0;
                for (int i = lane; i < per; i += 64) {
                    const uint32_t key = imp_key(imp[fb + i]);
                    gt += key > T; eq += key == T;
                }
                for (int o = 32; o > 0; o >>= 1) { gt += __shfl_xor(gt, o); eq += __shfl_xor(eq, o); }
                if (lane == 0) { s_gt[j] = gt; s_eq[j] = eq; }
            }
        }
        __syncthreads();
        // inclusive scan of eq over the chunk
        int cur = 0;
        if ((uint32_t)tid < nf) s_scan[0][tid] = s_eq[tid];
        __syncthreads();
        for (uint32_t d = 1; d < nf; d <<= 1) {
            if ((uint32_t)tid < nf) {
                uint32_t v = s_scan[cur][tid];
                if ((uint32_t)tid >= d) v += s_scan[cur][tid - d];    // at most n < 2^32 in total: no overflow
                s_scan[cur ^ 1][tid] = v;
            }
            cur ^= 1;
            __syncthreads();
        }
        if ((uint32_t)tid < nf) {
            const uint32_t eq = s_eq[tid], before = s_scan[cur][tid] - eq;
            const uint32_t room = before < left ? left - before : 0u;
            const uint32_t ties = eq < room ? eq : room;
            frame_nsel[c0 + tid] = s_gt[tid] + ties; frame_ties[c0 + tid] = ties;
        }
        const uint32_t tot = s_scan[cur][nf - 1];
        left = tot < left ? left - tot : 0u;
        __syncthreads();
    }
}

// Exclusive prefix count of a predicate over a 256-thread workgroup, in thread order.
__device__ __forceinline__ uint32_t block_prefix256(bool pred, uint32_t* s_w /*[4]*/, uint32_t& total)
{
    const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
    unsigned long long m = __ballot(pred);
    uint32_t pre = __popcll(m & ((1ull << lane) - 1ull));
    __syncthreads();                       // s_w free for reuse
    if (lane == 0) s_w[w] = __popcll(m);
    __syncthreads();
    uint32_t off = 0; total = 0;
    for (int i = 0; i < 4; ++i) { uint32_t c = s_w[i]; if (i < w) off += c; total += c; }
    return pre + off;
}

// Kernel 2: one workgroup per frame writes the frame's mask and its slice of the list.
__global__ __launch_bounds__(256) void k_select_write(const float* __restrict__ imp,
                                                      const int32_t* __restrict__ frame_seg,
                                                      const uint32_t* __restrict__ seg_T,
                                                      const uint32_t* __restrict__ frame_nsel,
                                                      const uint32_t* __restrict__ frame_ties,
                                                      int per, int F, uint8_t* __restrict__ mask,
                                                      uint32_t* __restrict__ list,
                                                      uint32_t* __restrict__ n_sel)
{
    __shared__ uint32_t s_w[4];
    __shared__ uint32_t s_base;
    const int tid = threadIdx.x, f = blockIdx.x;
    if (tid == 0) s_base = 0;
    __syncthreads();
    uint32_t local = 0;
    for (int i = tid; i < f; i += 256) if (frame_seg[i] >= 0) local += frame_nsel[i];
    if (local) atomicAdd(&s_base, local);
    __syncthreads();
    const uint32_t base = s_base;
    const int seg = frame_seg[f];
    const size_t fb = (size_t)f * per;
    if (seg < 0) {
        for (int i = tid; i < per; i += 256) mask[fb + i] = 0;
        if (f == F - 1 && tid == 0) *n_sel = base;
        return;
    }
    const uint32_t T = seg_T[seg], ties_allowed = frame_ties[f];
    uint32_t run_sel = 0, run_eq = 0;
    for (int c = 0; c < per; c += 256) {
        const int i = c + tid;
        const bool valid = i < per;
        const uint32_t key = valid ? imp_key(imp[fb + i]) : 0u;
        const bool gt = valid && key > T, eq = valid && key == T;
        uint32_t tot_eq, tot_sel;
        uint32_t eq_pre = block_prefix256(eq, s_w, tot_eq);
        const bool sel = gt || (eq && (run_eq + eq_pre) < ties_allowed);
        uint32_t sel_pre = block_prefix256(sel, s_w, tot_sel);
        if (valid) {
            mask[fb + i] = sel ? 1 : 0;
            if (sel) list[base + run_sel + sel_pre] = (uint32_t)(fb + i);
        }
        run_eq += tot_eq; run_sel += tot_sel;
    }
    if (f == F - 1 && tid == 0) *n_sel = base + run_sel;
}

// Segment tables travel as kernel arguments (copied at launch), so the caller's array may be
// freed as soon as rh_select_regions returns and no host synchronisation is needed.
struct seg_chunk { uint32_t n, first; uint32_t fb[64], fe[64], k[64], thr[64]; };

// One workgroup.  The first chunk of a call (c.first == 0) also marks every frame as belonging to
// no segment before the segments' frames are labelled.
__global__ __launch_bounds__(256) void k_upload_segments(seg_chunk c, int per, int F, uint32_t* __restrict__ seg_par,
                                                         int32_t* __restrict__ frame_seg)
{
    if (c.first == 0) {
        for (int f = threadIdx.x; f < F; f += 256) frame_seg[f] = -1;
        __syncthreads();
    }
    for (uint32_t s = 0; s < c.n; ++s) {
        if (threadIdx.x == 0) {
            uint32_t* p = seg_par + 4 * (size_t)(c.first + s);
            p[0] = c.fb[s] * (uint32_t)per; p[1] = c.fe[s] * (uint32_t)per; p[2] = c.k[s]; p[3] = c.thr[s];
        }
        for (uint32_t f = c.fb[s] + threadIdx.x; f < c.fe[s]; f += 256) frame_seg[f] = (int32_t)(c.first + s);
    }
}

hipError_t rh_enqueue_select(hipStream_t stream, const rh_select_scratch& sc, const float* imp, int F, int per,
                                 const rh_segment* segs, int nseg, int mode, uint8_t* mask, uint32_t* list, uint32_t* n_sel)
{
    for (int s0 = 0; s0 < nseg || s0 == 0; s0 += 64) {       // at least one launch: it clears frame_seg
        seg_chunk c;
        c.n = (uint32_t)((nseg - s0) < 64 ? (nseg - s0) : 64); c.first = (uint32_t)s0;
        for (uint32_t i = 0; i < c.n; ++i) {
            const rh_segment& g = segs[s0 + i];
            c.fb[i] = g.frame_begin; c.fe[i] = g.frame_end; c.k[i] = g.k; memcpy(&c.thr[i], &g.thr, 4);
        }
        hipLaunchKernelGGL(k_upload_segments, dim3(1), dim3(256), 0, stream, c, per, F, sc.seg_par, sc.frame_seg);
    }
    if (nseg > 0)
        hipLaunchKernelGGL(k_select_kth, dim3(nseg), dim3(1024), 0, stream, imp, sc.seg_par, mode, per, sc.seg_T,
                           sc.frame_nsel, sc.frame_ties);
    hipLaunchKernelGGL(k_select_write, dim3(F), dim3(256), 0, stream, imp, sc.frame_seg, sc.seg_T, sc.frame_nsel,
                       sc.frame_ties, per, F, mask, list, n_sel);
    return hipGetLastError();
}

// Argument checks shared by both entry points; returns a message or null.
const char* rh_check_select_args(const float* importance, int F, const rh_segment* segs, int nseg, int mode,
                                     const uint8_t* mask, const uint32_t* list, const uint32_t* n_sel, rh_status* st)
{
    *st = RH_E_INVALID;
    if (!importance || !mask || !list || !n_sel || (nseg > 0 && !segs) || nseg < 0) return "null argument";
    if (mode != RH_TOPK && mode != RH_THRESHOLD) return "bad mode";
    if (nseg > F) return "more segments than frames";
    uint32_t prev_end = 0;
    for (int s = 0; s < nseg; ++s) {
        const rh_segment& g = segs[s];
        if (g.frame_begin > g.frame_end || g.frame_end > (uint32_t)F || g.frame_begin < prev_end)
            return "a segment is out of range, unordered or overlapping";
        prev_end = g.frame_end;
    }
    *st = RH_OK;
    return nullptr;
}

rh_status rh_launch_select(rh_ctx* ctx, const float* imp, int F, const rh_segment* segs, int nseg, int mode,
                           uint8_t* mask, uint32_t* list, uint32_t* n_sel)
{
    rh_status st;
    if (const char* msg = rh_check_select_args(imp, F, segs, nseg, mode, mask, list, n_sel, &st))
        RH_FAIL(ctx, st, "rh_select_regions: %s", msg);
    const int n_up = nseg > 0 ? (nseg + 63) / 64 : 1;
    rh_prof_scope ps(ctx, RH_PROF_SELECT, n_up + (nseg > 0 ? 2 : 1));
    const rh_select_scratch sc = {ctx->frame_seg, ctx->seg_par, ctx->seg_T, ctx->frame_nsel, ctx->frame_ties};
    RH_HIP(ctx, rh_enqueue_select(ctx->stream, sc, imp, F, ctx->per, segs, nseg, mode, mask, list, n_sel));
    return RH_OK;
}


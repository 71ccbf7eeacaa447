// C ABI of librh.so: argument validation, context and scratch management, and the order in
// which the kernels of each call are enqueued.  No arithmetic of the method lives here.
#include <string.h>

#include <new>

#include "rh_internal.h"

static bool build_layers(const rh_net_desc& d, std::vector<rh_layer>& L, size_t& n_floats)
{
    const int C = d.channels, s = d.scale;
    std::vector<std::pair<int, int>> io;
    if (C < 1 || C > 1024 || s < 1 || s > 4) return false;
    if (d.topology == RH_NET_PLAIN) {
        if (d.n_blocks < 2) return false;
        io.push_back({3, C});
        for (int i = 0; i < d.n_blocks - 2; ++i) io.push_back({C, C});
        io.push_back({C, 3 * s * s});
    } else if (d.topology == RH_NET_RES || d.topology == RH_NET_EDSR) {
        if (d.n_blocks < 0) return false;
        io.push_back({3, C});
        for (int i = 0; i < 2 * d.n_blocks; ++i) io.push_back({C, C});
        if (d.topology == RH_NET_RES) io.push_back({C, 3 * s * s});
        else {
            io.push_back({C, C});
            if (s == 2 || s == 3) io.push_back({C, C * s * s});
            else if (s == 4) { io.push_back({C, 4 * C}); io.push_back({C, 4 * C}); }
            else return false;
            io.push_back({C, 3});
        }
    } else return false;
    size_t off = 0;
    for (auto& p : io) {
        rh_layer l{};
        l.cin = p.first; l.cout = p.second; l.w_off = off; off += (size_t)l.cout * 9 * l.cin;
        l.b_off = off; off += l.cout; l.ps = 1;
        L.push_back(l);
    }
    n_floats = off;
    return true;
}

extern "C" uint32_t rh_budget(uint32_t bin_h, uint32_t bin_w, uint32_t n_bins)
{
    return (uint32_t)(((uint64_t)bin_h * bin_w * n_bins) / (RH_MB * RH_MB));
}

extern "C" const char* rh_last_error(const rh_ctx* ctx) { return ctx ? ctx->err : "null context"; }

template <typename T> static hipError_t dalloc(T** p, size_t n) { return hipMalloc((void**)p, (n ? n : 1) * sizeof(T)); }

extern "C" void rh_destroy(rh_ctx* ctx)
{
    if (!ctx) return;
    (void)hipStreamSynchronize(ctx->stream);
    for (rh_prof_rec& r : ctx->prof_pending) { if (r.t0) (void)hipEventDestroy(r.t0); if (r.t1) (void)hipEventDestroy(r.t1); }
    for (hipEvent_t e : ctx->prof_pool) (void)hipEventDestroy(e);
    void* ptrs[] = {ctx->w_f32, ctx->wpack, ctx->bpack, ctx->fold_w, ctx->fold_b, ctx->frame_seg, ctx->seg_par, ctx->seg_T, ctx->seg_budget,
                    ctx->frame_nsel, ctx->frame_ties, ctx->owner_id, ctx->rank_of_id, ctx->raw, ctx->sorted,
                    ctx->pcount, ctx->tr_off, ctx->tr_A, ctx->tr_T, ctx->act,
                    ctx->cell_mark, ctx->cell_live, ctx->cell_dead, ctx->cell_cnt, ctx->need_dmin, ctx->need_lists, ctx->need_cnt};
    for (void* p : ptrs) if (p) (void)hipFree(p);
    delete ctx;
}

extern "C" rh_status rh_create(const rh_config* cfg, const float* weights, size_t n_floats, void* hip_stream,
                               rh_ctx** out)
{
    if (!cfg || !weights || !out) return RH_E_INVALID;
    *out = nullptr;
    if (cfg->frame_w < 16 || cfg->frame_h < 16) return RH_E_SHAPE;
    if (cfg->frame_w > 16 * 4095 || cfg->frame_h > 16 * 4095) return RH_E_SHAPE;
    if (cfg->max_frames < 1 || cfg->max_bins < 1 || cfg->max_bins >= (int)RH_NO_BIN) return RH_E_SHAPE;
    if (cfg->halo < 0 || cfg->bin_size < 16 || cfg->bin_size % 4 || cfg->bin_size > 4096) return RH_E_SHAPE;
    if (RH_MB + 2 * cfg->halo > cfg->bin_size) return RH_E_SHAPE;
    if (cfg->connectivity != 4 && cfg->connectivity != 8) return RH_E_INVALID;
    if (cfg->sort_policy != RH_SORT_DENSITY && cfg->sort_policy != RH_SORT_AREA) return RH_E_INVALID;
    if (cfg->rotate != 0 && cfg->rotate != 1) return RH_E_INVALID;
    if (cfg->per_layer_tail != 0 && cfg->per_layer_tail != 1) return RH_E_INVALID;
    if (cfg->precision != RH_FP32 && cfg->precision != RH_BF16) return RH_E_INVALID;
    const int Tmax = (cfg->bin_size - 2 * cfg->halo) / RH_MB;
    if (cfg->max_box_mbs < 0 || cfg->max_box_mbs > Tmax || Tmax > 255) return RH_E_SHAPE;
    rh_ctx* ctx = new (std::nothrow) rh_ctx();
    if (!ctx) return RH_E_NOMEM;
    ctx->cfg = *cfg; ctx->stream = (hipStream_t)hip_stream; ctx->err[0] = 0;
    // a partial macroblock at the right / bottom edge counts as one
    ctx->mbw = (cfg->frame_w + RH_MB - 1) / RH_MB; ctx->mbh = (cfg->frame_h + RH_MB - 1) / RH_MB; ctx->per = ctx->mbw * ctx->mbh;
    ctx->T = cfg->max_box_mbs ? cfg->max_box_mbs : Tmax;
    size_t need = 0;
    if (!build_layers(cfg->net, ctx->layers, need) || need != n_floats) { delete ctx; return RH_E_SHAPE; }
    // LDS limits of the planning kernels: 16 B per macroblock of a frame; 12 B per free rectangle
    const int side = RH_MB + 2 * cfg->halo, per_bin = (cfg->bin_size / side) * (cfg->bin_size / side);
    long fc = (long)cfg->max_bins * per_bin + 2;
    ctx->free_cap = (int)(fc < 12000 ? fc : 12000);
    if ((size_t)ctx->per * 16 > 150 * 1024) { delete ctx; return RH_E_SHAPE; }
    const size_t total = (size_t)ctx->per * cfg->max_frames;
    if (total > 0x7FFFFFFFu) { delete ctx; return RH_E_SHAPE; }
    rh_status st = RH_OK;
    hipError_t e = hipGetDevice(&ctx->device);
#define A(call) if (e == hipSuccess) e = (call)
    if (e == hipSuccess && (ctx->device < 0 || ctx->device >= RH_MAX_DEVICES)) { delete ctx; return RH_E_DEVICE; }
    A(hipDeviceGetAttribute(&ctx->n_cu, hipDeviceAttributeMultiprocessorCount, ctx->device));
    if (e == hipSuccess && ctx->n_cu < 1) ctx->n_cu = 1;
    A(dalloc(&ctx->w_f32, n_floats));
    A(hipMemcpy(ctx->w_f32, weights, n_floats * sizeof(float), hipMemcpyHostToDevice));
    A(dalloc(&ctx->frame_seg, cfg->max_frames)); A(dalloc(&ctx->seg_par, 4 * (size_t)cfg->max_frames));
    A(dalloc(&ctx->seg_T, cfg->max_frames)); A(dalloc(&ctx->seg_budget, cfg->max_frames));
    A(dalloc(&ctx->frame_nsel, cfg->max_frames)); A(dalloc(&ctx->frame_ties, cfg->max_frames));
    A(dalloc(&ctx->owner_id, total)); A(dalloc(&ctx->rank_of_id, total));
    A(dalloc(&ctx->raw, total)); A(dalloc(&ctx->sorted, total));
    A(dalloc(&ctx->pcount, 8 + 2 * total));
    A(dalloc(&ctx->tr_off, (size_t)cfg->max_frames + 1)); A(dalloc(&ctx->tr_A, cfg->max_frames)); A(dalloc(&ctx->tr_T, cfg->max_frames));
#undef A
    if (e != hipSuccess) {
        snprintf(ctx->err, sizeof(ctx->err), "rh_create: %s", hipGetErrorString(e));
        st = (e == hipErrorOutOfMemory) ? RH_E_NOMEM : RH_E_DEVICE;
    }
    if (st == RH_OK) st = rh_plan_init(ctx);
    if (st == RH_OK && cfg->precision == RH_BF16 && cfg->net.channels == 64) st = rh_mask_init(ctx);
    if (st == RH_OK && cfg->precision == RH_BF16) st = rh_pack_weights_bf16(ctx, weights);
    if (st == RH_OK && cfg->precision == RH_BF16 && !cfg->per_layer_tail) st = rh_fold_weights(ctx, weights);
    if (st != RH_OK) { rh_destroy(ctx); return st; }
    *out = ctx;
    return RH_OK;
}

static hipEvent_t prof_event(rh_ctx* ctx)
{
    hipEvent_t e = nullptr;
    if (!ctx->prof_pool.empty()) { e = ctx->prof_pool.back(); ctx->prof_pool.pop_back(); }
    else if (hipEventCreate(&e) != hipSuccess) e = nullptr;
    return e;
}

void rh_prof_begin(rh_ctx* ctx, int cls)
{
    if (!ctx->prof_on) return;
    rh_prof_rec r{cls, 0, prof_event(ctx), prof_event(ctx)};
    if (r.t0) (void)hipEventRecord(r.t0, ctx->stream);
    ctx->prof_pending.push_back(r);
}

void rh_prof_end(rh_ctx* ctx, uint32_t launches)
{
    if (!ctx->prof_on || ctx->prof_pending.empty()) return;
    rh_prof_rec& r = ctx->prof_pending.back();
    r.launches = launches;
    if (r.t1) (void)hipEventRecord(r.t1, ctx->stream);
}

extern "C" rh_status rh_profile_enable(rh_ctx* ctx, int32_t on)
{
    if (!ctx) return RH_E_INVALID;
    ctx->prof_on = on != 0;
    return RH_OK;
}

extern "C" rh_status rh_profile_read(rh_ctx* ctx, double* ms, uint32_t* launches)
{
    if (!ctx) return RH_E_INVALID;
    if (!ms || !launches) RH_FAIL(ctx, RH_E_INVALID, "rh_profile_read: null argument");
    RH_HIP(ctx, hipStreamSynchronize(ctx->stream));
    for (rh_prof_rec& r : ctx->prof_pending) {
        float t = 0.f;
        if (r.t0 && r.t1 && hipEventElapsedTime(&t, r.t0, r.t1) == hipSuccess) {
            ctx->prof_ms[r.cls] += t; ctx->prof_launches[r.cls] += r.launches;
        }
        if (r.t0) ctx->prof_pool.push_back(r.t0);
        if (r.t1) ctx->prof_pool.push_back(r.t1);
    }
    ctx->prof_pending.clear();
    for (int i = 0; i < RH_PROF_N; ++i) { ms[i] = ctx->prof_ms[i]; launches[i] = ctx->prof_launches[i]; ctx->prof_ms[i] = 0; ctx->prof_launches[i] = 0; }
    return RH_OK;
}

extern "C" rh_status rh_set_stream(rh_ctx* ctx, void* hip_stream)
{
    if (!ctx) return RH_E_INVALID;
    ctx->stream = (hipStream_t)hip_stream;
    return RH_OK;
}

rh_status rh_ensure_workspace(rh_ctx* ctx, size_t bytes)
{
    if (bytes <= ctx->act_bytes) return RH_OK;
    RH_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (ctx->act) { (void)hipFree(ctx->act); ctx->act = nullptr; ctx->act_bytes = 0; }
    hipError_t e = hipMalloc(&ctx->act, bytes);
    if (e != hipSuccess) RH_FAIL(ctx, RH_E_NOMEM, "workspace of %zu bytes: %s", bytes, hipGetErrorString(e));
    ctx->act_bytes = bytes;
    return RH_OK;
}

extern "C" rh_status rh_select_regions(rh_ctx* ctx, const float* importance, int32_t F, const rh_segment* segs,
                                       int32_t nseg, int32_t mode, uint8_t* mask, uint32_t* list, uint32_t* n_sel)
{
    if (!ctx) return RH_E_INVALID;
    if (F < 1 || F > ctx->cfg.max_frames) RH_FAIL(ctx, RH_E_CAPACITY, "rh_select_regions: F=%d outside [1,%d]", F, ctx->cfg.max_frames);
    return rh_launch_select(ctx, importance, F, segs, nseg, mode, mask, list, n_sel);
}

extern "C" rh_status rh_temporal_phi(rh_ctx* ctx, const int16_t* res_y, int32_t F, int32_t tau, int32_t min_area,
                                     uint64_t* phi)
{
    if (!ctx) return RH_E_INVALID;
    if (!res_y || !phi) RH_FAIL(ctx, RH_E_INVALID, "rh_temporal_phi: null argument");
    if (F < 1 || F > ctx->cfg.max_frames) RH_FAIL(ctx, RH_E_CAPACITY, "rh_temporal_phi: F=%d outside [1,%d]", F, ctx->cfg.max_frames);
    if (tau < 0 || min_area < 1) RH_FAIL(ctx, RH_E_INVALID, "rh_temporal_phi: tau=%d must be >= 0 and min_area=%d >= 1", tau, min_area);
    return rh_launch_temporal_phi(ctx, res_y, F, tau, min_area, phi);
}

extern "C" rh_status rh_temporal_select(rh_ctx* ctx, const uint64_t* phi, const int32_t* stream_off, int32_t n_streams,
                                        int32_t n_total, uint32_t* alloc, uint8_t* selected, uint32_t* reuse_from,
                                        uint32_t* n_selected)
{
    if (!ctx) return RH_E_INVALID;
    if (!phi || !stream_off || !alloc || !selected || !reuse_from || !n_selected)
        RH_FAIL(ctx, RH_E_INVALID, "rh_temporal_select: null argument");
    if (n_streams < 1 || n_streams > 1024) RH_FAIL(ctx, RH_E_CAPACITY, "rh_temporal_select: %d streams outside [1,1024]", n_streams);
    if (n_total < n_streams || n_total > 65535)
        RH_FAIL(ctx, RH_E_INVALID, "rh_temporal_select: a budget of %d frames is outside [%d streams, 65535]", n_total, n_streams);
    if (stream_off[0] != 0) RH_FAIL(ctx, RH_E_INVALID, "rh_temporal_select: stream_off[0] must be 0");
    for (int s = 0; s < n_streams; ++s) {
        const long n = (long)stream_off[s + 1] - stream_off[s];
        if (n < 1 || n > 2048) RH_FAIL(ctx, RH_E_INVALID, "rh_temporal_select: stream %d has %ld frames, outside [1,2048]", s, n);
    }
    const int F = stream_off[n_streams];
    if (F > ctx->cfg.max_frames) RH_FAIL(ctx, RH_E_CAPACITY, "rh_temporal_select: %d frames exceed max_frames=%d", F, ctx->cfg.max_frames);
    // Phi <= 2^32 * (most blobs a frame can hold); all sums of changes must stay below 2^63
    const uint64_t blobs = (uint64_t)(ctx->cfg.frame_h / 2 + 1) * (uint64_t)(ctx->cfg.frame_w / 2 + 1);
    if ((uint64_t)F * blobs >= (1ull << 31))
        RH_FAIL(ctx, RH_E_SHAPE, "rh_temporal_select: %d frames of %dx%d could overflow the 64-bit sums", F, ctx->cfg.frame_w, ctx->cfg.frame_h);
    return rh_launch_temporal_select(ctx, phi, stream_off, n_streams, n_total, alloc, selected, reuse_from, n_selected);
}

extern "C" rh_status rh_temporal_spread(rh_ctx* ctx, float* importance, int32_t F, const uint8_t* selected,
                                        const uint32_t* reuse_from)
{
    if (!ctx) return RH_E_INVALID;
    if (!importance || !selected || !reuse_from) RH_FAIL(ctx, RH_E_INVALID, "rh_temporal_spread: null argument");
    if (F < 1 || F > ctx->cfg.max_frames) RH_FAIL(ctx, RH_E_CAPACITY, "rh_temporal_spread: F=%d outside [1,%d]", F, ctx->cfg.max_frames);
    return rh_launch_temporal_spread(ctx, importance, F, selected, reuse_from);
}

extern "C" rh_status rh_pack(rh_ctx* ctx, const uint8_t* frames, int32_t F, const float* importance,
                             const uint8_t* mask, const uint32_t* list, const uint32_t* n_sel, uint8_t* bins,
                             rh_box* boxes, rh_mbplace* places, uint32_t* counts)
{
    if (!ctx) return RH_E_INVALID;
    if (!frames || !importance || !mask || !list || !n_sel || !bins || !boxes || !places || !counts)
        RH_FAIL(ctx, RH_E_INVALID, "rh_pack: null argument");
    if (F < 1 || F > ctx->cfg.max_frames) RH_FAIL(ctx, RH_E_CAPACITY, "rh_pack: F=%d outside [1,%d]", F, ctx->cfg.max_frames);
    rh_status st = rh_launch_plan(ctx, F, importance, mask, list, n_sel, boxes, places, counts);
    if (st != RH_OK) return st;
    return rh_launch_gather(ctx, frames, F, boxes, counts, bins);
}

extern "C" rh_status rh_enhance(rh_ctx* ctx, const uint8_t* in, int32_t N, int32_t H, int32_t W, float* out,
                                const uint32_t* n_valid)
{
    if (!ctx) return RH_E_INVALID;
    if (!in || !out) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance: null argument");
    if (N < 1 || H < 3 || W < 3 || H > 16384 || W > 16384 || N > 65535) RH_FAIL(ctx, RH_E_SHAPE, "rh_enhance: bad shape N=%d H=%d W=%d", N, H, W);
    if ((uintptr_t)out & 15) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance: out must be 16-byte aligned");
    return ctx->cfg.precision == RH_BF16 ? rh_launch_enhance_bf16(ctx, in, N, H, W, out, n_valid)
                                         : rh_launch_enhance_fp32(ctx, in, N, H, W, out, n_valid);
}

extern "C" rh_status rh_enhance_exact(rh_ctx* ctx, const uint8_t* in, int32_t N, const rh_box* boxes,
                                      const uint32_t* counts, float* out, const uint32_t* n_valid)
{
    if (!ctx) return RH_E_INVALID;
    if (!in || !out || !boxes || !counts) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance_exact: null argument");
    if (N < 1 || N > 65535) RH_FAIL(ctx, RH_E_SHAPE, "rh_enhance_exact: bad N=%d", N);
    if ((uintptr_t)out & 15) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance_exact: out must be 16-byte aligned");
    const int S = ctx->cfg.bin_size;
    ctx->bz_boxes = boxes; ctx->bz_counts = counts;
    const rh_status st = ctx->cfg.precision == RH_BF16 ? rh_launch_enhance_bf16(ctx, in, N, S, S, out, n_valid)
                                                       : rh_launch_enhance_fp32(ctx, in, N, S, S, out, n_valid);
    ctx->bz_boxes = nullptr; ctx->bz_counts = nullptr;
    return st;
}

extern "C" rh_status rh_enhance_masked(rh_ctx* ctx, const uint8_t* in, int32_t N, const rh_box* boxes,
                                       const uint32_t* counts, float* out, const uint32_t* n_valid)
{
    if (!ctx) return RH_E_INVALID;
    if (!in || !out || !boxes || !counts) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance_masked: null argument");
    if (ctx->cfg.precision != RH_BF16 || ctx->cfg.net.channels != 64)
        RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "rh_enhance_masked: only bf16 networks with 64 channels have a tile-list conv kernel");
    if (N < 1 || N > ctx->cfg.max_bins) RH_FAIL(ctx, RH_E_CAPACITY, "rh_enhance_masked: N=%d outside [1,%d]", N, ctx->cfg.max_bins);
    if ((uintptr_t)out & 15) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance_masked: out must be 16-byte aligned");
    const int S = ctx->cfg.bin_size;
    ctx->mk_boxes = boxes; ctx->mk_counts = counts;
    const rh_status st = rh_launch_enhance_bf16(ctx, in, N, S, S, out, n_valid);
    ctx->mk_boxes = nullptr; ctx->mk_counts = nullptr;
    return st;
}

extern "C" rh_status rh_enhance_needed(rh_ctx* ctx, const uint8_t* in, int32_t N, const rh_mbplace* places,
                                       const uint32_t* counts, float* out, const uint32_t* n_valid)
{
    if (!ctx) return RH_E_INVALID;
    if (!in || !out || !places || !counts) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance_needed: null argument");
    if (ctx->cfg.precision != RH_BF16 || ctx->cfg.net.channels != 64)
        RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "rh_enhance_needed: only bf16 networks with 64 channels have a tile-list conv kernel");
    if (N < 1 || N > ctx->cfg.max_bins) RH_FAIL(ctx, RH_E_CAPACITY, "rh_enhance_needed: N=%d outside [1,%d]", N, ctx->cfg.max_bins);
    if ((uintptr_t)out & 15) RH_FAIL(ctx, RH_E_INVALID, "rh_enhance_needed: out must be 16-byte aligned");
    const int nb = rh_needed_radii(&ctx->cfg.net, ctx->cfg.per_layer_tail, ctx->nd_radii, RH_NEED_MAX_LAYERS);
    if (nb < 0)
        RH_FAIL(ctx, RH_E_UNIMPLEMENTED, "rh_enhance_needed: not with the upsampler run layer by layer (per_layer_tail), nor with more than %d layers",
                RH_NEED_MAX_LAYERS - 2);
    const int S = ctx->cfg.bin_size;
    ctx->nd_places = places; ctx->nd_counts = counts;
    const rh_status st = rh_launch_enhance_bf16(ctx, in, N, S, S, out, n_valid);
    ctx->nd_places = nullptr; ctx->nd_counts = nullptr;
    return st;
}

extern "C" rh_status rh_unpack(rh_ctx* ctx, const float* enhanced, int32_t n_img, int32_t ih, int32_t iw,
                               const rh_mbplace* places, const uint32_t* n_places, const uint8_t* frames_lr,
                               int32_t F, uint8_t* frames_hr, float* sel)
{
    if (!ctx) return RH_E_INVALID;
    if (!enhanced || !places || !n_places || !frames_lr || !frames_hr) RH_FAIL(ctx, RH_E_INVALID, "rh_unpack: null argument");
    if (F < 1 || F > ctx->cfg.max_frames) RH_FAIL(ctx, RH_E_CAPACITY, "rh_unpack: F=%d outside [1,%d]", F, ctx->cfg.max_frames);
    if (n_img < 1 || ih < RH_MB || iw < RH_MB) RH_FAIL(ctx, RH_E_SHAPE, "rh_unpack: bad enhanced shape");
    return rh_launch_unpack(ctx, enhanced, n_img, ih, iw, places, n_places, frames_lr, F, frames_hr, sel);
}

extern "C" rh_status rh_identity_places(rh_ctx* ctx, int32_t F, rh_mbplace* places, uint32_t* n_places)
{
    if (!ctx) return RH_E_INVALID;
    if (!places || !n_places) RH_FAIL(ctx, RH_E_INVALID, "rh_identity_places: null argument");
    if (F < 1 || F > ctx->cfg.max_frames) RH_FAIL(ctx, RH_E_CAPACITY, "rh_identity_places: F=%d outside [1,%d]", F, ctx->cfg.max_frames);
    return rh_launch_identity_places(ctx, F, places, n_places);
}

extern "C" rh_status rh_read_counts(rh_ctx* ctx, const uint32_t* counts, uint32_t out[4])
{
    if (!ctx) return RH_E_INVALID;
    if (!counts || !out) RH_FAIL(ctx, RH_E_INVALID, "rh_read_counts: null argument");
    RH_HIP(ctx, hipMemcpyAsync(out, counts, 4 * sizeof(uint32_t), hipMemcpyDeviceToHost, ctx->stream));
    RH_HIP(ctx, hipStreamSynchronize(ctx->stream));
    if (out[2]) RH_FAIL(ctx, RH_E_CAPACITY, "packing needs more than max_bins=%d bins", ctx->cfg.max_bins);
    return RH_OK;
}

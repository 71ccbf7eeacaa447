// Internal declarations shared by the HIP translation units of librh.so.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stdio.h>
#include <vector>

#include "rh.h"

#define RH_MB 16
#define RH_NO_BIN 0xFFFFu
// A cell-list entry (box-masked and needed-region modes): image n, cell row cy (rows of RH_CELL_H),
// cell column cx packed as n << 16 | cy << 7 | cx  (bin_size <= 4096: cy < 512, cx < 128; n < 65536),
// so that the kernels that walk a list decode an entry with shifts
#define RH_CELL_ENTRY(n, cy, cx) (((uint32_t)(n) << 16) | ((uint32_t)(cy) << 7) | (uint32_t)(cx))
#define RH_NEED_RMAX 63          // largest layer radius that has a cell list of its own (needed-region mode)
#define RH_NEED_MAX_LAYERS 512
#define RH_MAX_DEVICES 64     // device indexes a context may live on (per-device launch attributes)

struct rh_layer {
    int cin, cout;          // true channel counts
    size_t w_off, b_off;    // offsets (floats) into the fp32 blob
    // bf16 path: weights repacked into MFMA fragment order (see conv_mfma.hip)
    size_t wp_off;          // offset (bytes) into wpack
    size_t bp_off;          // offset (floats) into bpack (bias, permuted/padded like the weights)
    int cout_pad;           // cout rounded up to the kernel's M tile
    int ps;                 // pixel-shuffle factor folded into the output-channel order (1 = none)
    int tail3;              // 1: last conv with 3 outputs, packed for k_conv_tail3 (conv_tail.hip)
};

// Raw (unsorted) box written by the labelling kernel.
struct rh_rawbox {
    uint32_t frame;
    uint16_t mbx0, mby0;
    uint16_t wmb, hmb;
    uint32_t id;
    float sum;
    double key;
};

struct rh_prof_rec { int cls; uint32_t launches; hipEvent_t t0, t1; };

struct rh_ctx {
    rh_config cfg;
    // optional per-kernel-class event timing
    bool prof_on;
    std::vector<rh_prof_rec> prof_pending;
    std::vector<hipEvent_t> prof_pool;
    double prof_ms[RH_PROF_N];
    uint32_t prof_launches[RH_PROF_N];
    hipStream_t stream;
    int device;
    int n_cu;               // compute units of the device: the persistent conv kernels launch one workgroup each
    int mbw, mbh, per;      // macroblock grid of one frame
    int T;                  // partition size in MBs
    int free_cap;           // capacity of the free-rectangle list (entries)
    char err[256];

    std::vector<rh_layer> layers;
    float* w_f32;           // dev: the fp32 blob as given
    void* wpack;            // dev: bf16 weights in fragment order (RH_BF16 only)
    float* bpack;           // dev: biases matching wpack's channel order
    // EDSR-shaped nets, bf16: the upsampler and the last conv composed into one 5 x 5 conv (conv_fold.hip)
    void* fold_w;           // dev: bf16 weights [class 9][chunk][tap 25][k-step][lane][8]
    float* fold_b;          // dev: [class][chunk][32]
    int fold_chunks;        // 32-row chunks of the composed conv's 3*s*s outputs (0: no composed conv)
    int fold_rows, fold_ipc;   // valid rows per chunk, output rows i per chunk

    // select scratch (dev)
    int32_t* frame_seg;     // [max_frames] segment of each frame or -1
    uint32_t* seg_par;      // [max_frames][4] per segment: g_begin, g_end, k, thr bits
    uint32_t* seg_T;        // [max_frames] per segment: threshold key
    uint32_t* seg_budget;   // [max_frames] per segment: ties to take
    uint32_t* frame_nsel;   // [max_frames]
    uint32_t* frame_ties;   // [max_frames] ties this frame may take
    // plan scratch (dev)
    uint32_t* owner_id;     // [total MBs] id of the box owning each selected MB
    uint32_t* rank_of_id;   // [total MBs] sorted position of the box with that id
    rh_rawbox* raw;         // [total MBs]
    rh_rawbox* sorted;      // [total MBs]
    uint32_t* pcount;       // [8] plan counters: 0 n_raw boxes
    // temporal reuse scratch (dev)
    int32_t* tr_off;        // [max_frames + 1] first frame of each stream
    uint64_t* tr_A;         // [max_frames] cumulative change before each frame
    uint64_t* tr_T;         // [max_frames] total change of each stream
    // exact-border mode: the boxes of the bins being enhanced (set for the duration of one
    // rh_enhance_exact call, null otherwise)
    const rh_box* bz_boxes;
    const uint32_t* bz_counts;
    // box-masked mode: the boxes of the bins being enhanced (set for the duration of one
    // rh_enhance_masked call, null otherwise) and the cell scratch (64-channel bf16 nets only)
    const rh_box* mk_boxes;
    const uint32_t* mk_counts;
    int cells_x, cells_y;   // cells per bin row / column
    uint8_t* cell_mark;     // [max_bins * cells] 1 while a box touches the cell; all zero between calls
    uint32_t* cell_live;    // [max_bins * cells] live cells = tile indices of the body convs
    uint32_t* cell_dead;    // [max_bins * cells] the others
    uint32_t* cell_cnt;     // [2] entries of the two lists
    // needed-region mode: the placement rows of the bins being enhanced (set for the duration of one
    // rh_enhance_needed call, null otherwise), the radius of every layer, and the scratch
    const rh_mbplace* nd_places;
    const uint32_t* nd_counts;
    int nd_radii[RH_NEED_MAX_LAYERS];   // [0] first conv, [1 + c] bf16-output conv c, then 0 for the tail
    int nd_conv;            // bf16-output convs launched so far in the call
    uint32_t* need_dmin;    // [max_bins * cells] smallest distance of a cell to a placed macroblock; all "none" between calls
    uint32_t* need_lists;   // [RH_NEED_RMAX + 1][need_cap] cells at distance <= r
    uint32_t* need_cnt;     // [RH_NEED_RMAX + 1] their numbers
    size_t need_cap;
    int conv_parity;        // direction of the next bf16 conv's tile walk (alternates)
    // enhance workspace (grow-only)
    void* act;
    size_t act_bytes;
};

#define RH_FAIL(ctx, code, ...)                                           \
    do {                                                                  \
        if (ctx) snprintf((ctx)->err, sizeof((ctx)->err), __VA_ARGS__);   \
        return (code);                                                    \
    } while (0)

#define RH_HIP(ctx, call)                                                             \
    do {                                                                              \
        hipError_t e_ = (call);                                                       \
        if (e_ != hipSuccess)                                                         \
            RH_FAIL(ctx, RH_E_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_)); \
    } while (0)

// kernels' host launchers (each returns after enqueueing)
// The selection's scratch memory: per-frame and per-segment tables of at least F entries each
// (seg_par: 4 per segment; there are at most F segments).
struct rh_select_scratch { int32_t* frame_seg; uint32_t *seg_par, *seg_T, *frame_nsel, *frame_ties; };
hipError_t rh_enqueue_select(hipStream_t stream, const rh_select_scratch& sc, const float* imp, int F, int per,
                             const rh_segment* segs, int nseg, int mode, uint8_t* mask, uint32_t* list, uint32_t* n_sel);
const char* rh_check_select_args(const float* importance, int F, const rh_segment* segs, int nseg, int mode,
                                 const uint8_t* mask, const uint32_t* list, const uint32_t* n_sel, rh_status* st);
rh_status rh_launch_select(rh_ctx*, const float* imp, int F, const rh_segment* segs, int nseg, int mode,
                           uint8_t* mask, uint32_t* list, uint32_t* n_sel);
rh_status rh_launch_plan(rh_ctx*, int F, const float* imp, const uint8_t* mask,
                         const uint32_t* list, const uint32_t* n_sel,
                         rh_box* boxes, rh_mbplace* places, uint32_t* counts);
rh_status rh_launch_gather(rh_ctx*, const uint8_t* frames, int F, const rh_box* boxes,
                           const uint32_t* counts, uint8_t* bins);
rh_status rh_launch_enhance_fp32(rh_ctx*, const uint8_t* in, int N, int H, int W, float* out,
                                 const uint32_t* n_valid);
rh_status rh_launch_enhance_bf16(rh_ctx*, const uint8_t* in, int N, int H, int W, float* out,
                                 const uint32_t* n_valid);
rh_status rh_launch_unpack(rh_ctx*, const float* enh, int n_img, int ih, int iw,
                           const rh_mbplace* places, const uint32_t* n_places,
                           const uint8_t* lr, int F, uint8_t* hr, float* sel);
rh_status rh_launch_identity_places(rh_ctx*, int F, rh_mbplace* places, uint32_t* n_places);
rh_status rh_launch_temporal_phi(rh_ctx*, const int16_t* res, int F, int tau, int min_area, uint64_t* phi);
rh_status rh_launch_temporal_select(rh_ctx*, const uint64_t* phi, const int32_t* stream_off, int n_streams,
                                    int n_total, uint32_t* alloc, uint8_t* selected, uint32_t* reuse_from,
                                    uint32_t* n_selected);
rh_status rh_launch_temporal_spread(rh_ctx*, float* imp, int F, const uint8_t* selected, const uint32_t* reuse_from);
rh_status rh_pack_weights_bf16(rh_ctx*, const float* host_blob);
rh_status rh_fold_weights(rh_ctx*, const float* host_blob);
rh_status rh_plan_init(rh_ctx*);
rh_status rh_mask_init(rh_ctx*);
// box-masked mode: the cell lists of the call in progress; zeros over the dead cells of three
// [N][S][S][64] bf16 tensors
rh_status rh_launch_cell_lists(rh_ctx*, int N, const uint32_t* n_valid, void* act0, void* act1, void* act2);
// needed-region mode: the per-radius cell lists of the call in progress
rh_status rh_launch_need_lists(rh_ctx*, int N, const uint32_t* n_valid);
extern "C" int32_t rh_needed_radii(const rh_net_desc* net, int32_t per_layer_tail, int32_t* radii, int32_t cap);
// exact-border mode: zero the out-of-frame part of every box in an activation tensor
// [N][S*res][S*res][px_bytes]; a no-op unless an rh_enhance_exact call is in progress
rh_status rh_zero_outside(rh_ctx*, void* act, int px_bytes, int res, int N, const uint32_t* n_valid);
void rh_fill_i32(rh_ctx*, int32_t* p, int32_t v, size_t n);
rh_status rh_ensure_workspace(rh_ctx*, size_t bytes);

// Event bracket around the launches of one kernel class (no-ops unless profiling is on).
void rh_prof_begin(rh_ctx*, int cls);
void rh_prof_end(rh_ctx*, uint32_t launches);
struct rh_prof_scope {
    rh_ctx* c; uint32_t n;
    rh_prof_scope(rh_ctx* ctx, int cls, uint32_t launches = 1) : c(ctx), n(launches) { rh_prof_begin(c, cls); }
    ~rh_prof_scope() { rh_prof_end(c, n); }
};

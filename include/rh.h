/*
 * rh.h - C ABI of the region-aware enhancer for AMD MI355X (gfx950).
 *
 * The path is the one RegenHance (arXiv 2407.16990) speeds up, Sec. 3.3:
 *   select   important 16x16 macroblocks (MBs) across all streams of a batch  (Sec. 3.3.1)
 *   pack     plan (Alg. 1, region-aware bin packing) + stitch pixels into bins (Sec. 3.3.2-3.3.3)
 *   enhance  run the super-resolution network on the packed bins only         (Sec. 3.3.3)
 *   unpack   paste enhanced MBs into the bilinearly interpolated frames        (Sec. 3.2.1, 3.3.3)
 *
 * General conventions
 *   - "dev" pointers are HIP device memory on the context's device, "host" pointers are
 *     ordinary host memory.  The caller owns every data buffer; the library never frees or
 *     reallocates them.  The context owns a copy of the weights and its scratch memory.
 *   - All work is enqueued on the context's HIP stream and the calls return after argument
 *     validation; only rh_read_counts and rh_create/rh_destroy synchronise.
 *   - Every call returns an rh_status; nothing aborts or throws across the ABI.  Argument
 *     errors are detected before any launch and leave outputs untouched.  rh_last_error gives
 *     a text for the last failure on that context.
 *   - One context serves one stream at a time; calls on one context must not overlap.
 *   - Tensors are dense, row-major, channels last: frames u8 [F][H][W][3].
 *   - Flat macroblock index g = (f*MBH + y)*MBW + x with MBW = ceil(W/16), MBH = ceil(H/16); f counts the
 *     (stream, frame) pairs of the batch in the caller's order (the MB index of Sec. 3.3.1).
 */
#ifndef RH_H
#define RH_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct rh_ctx rh_ctx;

typedef enum {
    RH_OK = 0,
    RH_E_INVALID = 1,       /* null pointer, bad enum, malformed segment list            */
    RH_E_SHAPE = 2,         /* sizes that the configuration or the kernels cannot take   */
    RH_E_CAPACITY = 3,      /* more bins/frames/images than the configured capacity      */
    RH_E_DEVICE = 4,        /* a HIP call failed                                         */
    RH_E_NOMEM = 5,
    RH_E_STATE = 6,
    RH_E_UNIMPLEMENTED = 7
} rh_status;

enum { RH_FP32 = 0, RH_BF16 = 1 };                   /* rh_config.precision              */
enum { RH_NET_PLAIN = 0, RH_NET_RES = 1, RH_NET_EDSR = 2 };
enum { RH_TOPK = 0, RH_THRESHOLD = 1 };              /* rh_select_regions mode           */
enum { RH_SORT_DENSITY = 0, RH_SORT_AREA = 1 };      /* rh_config.sort_policy            */

/*
 * The SR network (Sec. 3.3.3 only says "pre-trained EDSR"; the topologies are this build's).
 * All convolutions are 3x3, stride 1, zero padding at the tensor border, with bias.
 *   RH_NET_PLAIN: n_blocks convs (>= 2): 3->C ReLU, (n_blocks-2) x [C->C ReLU], C->3*s*s, shuffle s
 *   RH_NET_RES  : 3->C, n_blocks x [x + conv(ReLU(conv(x)))], C->3*s*s, shuffle s
 *   RH_NET_EDSR : 3->C (=h), n_blocks residual blocks, C->C then + h,
 *                 s=2,3: C->C*s*s, shuffle s;  s=4: two (C->4C, shuffle 2) stages;  then C->3
 * Pixel shuffle by r: out[y*r+i][x*r+j][c] = in[y][x][c*r*r + i*r + j].
 * The input is u8/255.  Weight blob (host, fp32): for each conv in the order above,
 * w[cout][ky][kx][cin] followed by b[cout].  With RH_BF16 the weights are rounded to bf16
 * (nearest even) at rh_create, activations are stored as bf16 between layers and every
 * convolution accumulates in fp32; with RH_FP32 everything is fp32.
 */
typedef struct { int32_t topology, channels, n_blocks, scale; } rh_net_desc;

typedef struct {
    int32_t frame_w, frame_h;   /* >= 16; MB grid = ceil(w/16) x ceil(h/16): a partial MB at
                                   the right / bottom edge is one MB, zero-filled when packed,
                                   and only its in-frame part is pasted                     */
    int32_t max_frames;         /* capacity F of one batch                                 */
    int32_t halo;               /* pixels of context added on each side of a box           */
    int32_t bin_size;           /* bins are bin_size x bin_size pixels (multiple of 4)     */
    int32_t max_bins;           /* capacity; more are reported as overflow                 */
    int32_t connectivity;       /* 4 or 8: neighbourhood for connected regions             */
    int32_t max_box_mbs;        /* Partition's preset size in MBs; 0 = (bin_size-2*halo)/16 */
    int32_t precision;          /* RH_FP32 | RH_BF16                                       */
    rh_net_desc net;
    int32_t sort_policy;        /* packing order (Alg. 1, Sort): RH_SORT_DENSITY = importance
                                   density first (the paper's), RH_SORT_AREA = the classic
                                   large-item-first order it is compared with (Sec. 3.3.2);
                                   ties: ascending box id                                   */
    int32_t rotate;             /* 1: RotatePacking (Alg. 1): a free area also takes a box
                                   turned by a quarter - stored with rows and columns
                                   exchanged - when it does not fit upright.  A conv net is
                                   not equivariant under that, so the enhanced pixels of a
                                   turned box differ from the upright ones (the paper accepts
                                   this); 0 keeps every box upright                         */
    int32_t per_layer_tail;     /* RH_BF16, RH_NET_EDSR only.  After the body these nets are linear
                                   (upsampling convs, pixel shuffles, last conv, no activation), so
                                   rh_enhance runs that part as ONE composed convolution (5 x 5 taps
                                   on the body's output, 3*s*s outputs, weights composed at rh_create):
                                   the same function without the high-resolution intermediate
                                   tensors and their bf16 rounding.  1: run these layers one by one
                                   instead (what rh_enhance_exact always does)                */
} rh_config;

/* One selection segment: frames [frame_begin, frame_end).  RH_TOPK uses k, RH_THRESHOLD thr. */
typedef struct { uint32_t frame_begin, frame_end, k; float thr; } rh_segment;

/* A placed box (Alg. 1): MB rectangle (mbx0, mby0, wmb, hmb) of frame `frame`, packed with its
 * halo at pixel (bx, by) of bin `bin`; id = smallest flat index of the MBs it owns.
 * rot = 1 (only with rh_config.rotate): the box is stored turned, bin pixel (bx + i, by + j) =
 * box pixel (column j, row i), and occupies (16*hmb + 2*halo) x (16*wmb + 2*halo) pixels.
 * bin = 0xFFFF marks a box that did not fit within max_bins. */
typedef struct {
    uint32_t frame;
    uint16_t mbx0, mby0;
    uint8_t wmb, hmb, rot, pad0;
    uint16_t bin, bx, by, pad1;
    uint32_t id;
} rh_box;                                             /* 24 bytes */

/* Where one selected MB lives: its 16x16 pixels start at (px, py) of bin `bin`; rot = 1: they
 * are stored with rows and columns exchanged (the MB belongs to a turned box). */
typedef struct { uint32_t mb_id, box; uint16_t bin, px, py, rot; } rh_mbplace;   /* 16 bytes */

/* Largest N with 256*N <= bin_h*bin_w*n_bins (Sec. 3.3.1, the MB budget). */
uint32_t rh_budget(uint32_t bin_h, uint32_t bin_w, uint32_t n_bins);

/*
 * Create a context on the current HIP device.  weights: host fp32 blob (layout above),
 * n_floats its length (checked against the descriptor).  hip_stream: a hipStream_t (NULL =
 * the default stream).  Allocates device scratch for the configured capacities.
 */
rh_status rh_create(const rh_config* cfg, const float* weights, size_t n_floats,
                    void* hip_stream, rh_ctx** out);
void rh_destroy(rh_ctx* ctx);
rh_status rh_set_stream(rh_ctx* ctx, void* hip_stream);
const char* rh_last_error(const rh_ctx* ctx);

/*
 * Cross-stream MB selection (Sec. 3.3.1).  importance: dev f32 [F][MBH][MBW].  segs: host
 * array of nseg segments, ascending and non-overlapping; frames outside every segment select
 * nothing.  RH_TOPK takes, per segment, the k most important MBs of the segment's queue
 * (importance descending; equal importance: lower flat index first; -0 = +0; NaN ranks last;
 * k is clipped to the segment size).  RH_THRESHOLD takes importance >= thr.
 * Outputs (dev): mask u8 [F][MBH][MBW] (0/1), list u32 (capacity F*MBH*MBW) = selected flat
 * indexes ascending, n_sel u32[1].
 */
rh_status rh_select_regions(rh_ctx* ctx, const float* importance, int32_t F,
                            const rh_segment* segs, int32_t nseg, int32_t mode,
                            uint8_t* mask, uint32_t* list, uint32_t* n_sel);

/*
 * Region-aware bin packing (Alg. 1) and stitching (Sec. 3.3.3).
 * Plan, on MB indexes only: connected regions of selected MBs per frame -> bounding boxes ->
 * boxes larger than max_box_mbs cut on a grid anchored at the box's top-left, each cell shrunk
 * to the region's own MBs inside it -> sort by importance density (fp32 sum of owned
 * importance in ascending flat index, divided in fp64 by the box area in MBs), highest first,
 * ties by id (rh_config.sort_policy selects large-item-first instead) -> first fit over an
 * ordered list of free rectangles; bins are opened on demand.
 * A box lands on the free rectangle's top-left; the L-shaped remainder becomes its larger
 * strip plus the rest, rectangles with a side < 16+2*halo are dropped, survivors replace the
 * free rectangle in the list, smaller area first.  Boxes stay upright (rot = 0) unless
 * rh_config.rotate is set.
 * Stitch: bins u8 [max_bins][S][S][3], 16-byte aligned; inside a placed box the frame's pixels (zero where the
 * halo leaves the frame), zero elsewhere; only bins [0, n_bins) are written.
 * Inputs (dev): frames u8 [F][H][W][3], importance, and mask/list/n_sel from rh_select_regions.
 * Outputs (dev): bins; boxes (capacity F*MBH*MBW) in placement order; places (same capacity)
 * in ascending mb_id; counts u32[4] = {n_boxes, n_bins, overflow, n_selected}.
 * If more than max_bins bins are needed, overflow = 1, n_bins = max_bins and the first box that
 * does not fit and all later ones carry bin = 0xFFFF (so do their MBs' places).
 */
rh_status rh_pack(rh_ctx* ctx, const uint8_t* frames, int32_t F, const float* importance,
                  const uint8_t* mask, const uint32_t* list, const uint32_t* n_sel,
                  uint8_t* bins, rh_box* boxes, rh_mbplace* places, uint32_t* counts);

/*
 * SR forward (Sec. 3.3.3) on N images u8 [N][H][W][3] -> raw network output f32
 * [N][s*H][s*W][3].  Used for the packed bins and, with whole frames, for the frame-based
 * comparison run.  n_valid (dev u32[1], may be NULL): when given, only images [0, *n_valid)
 * are computed (pass &counts[1] to avoid a host round trip).  H, W >= 3; out 16-byte aligned.
 * The context's activation workspace only grows: a call that needs more than every earlier call
 * synchronises the stream and reallocates it (sized by N, not by *n_valid); later calls of the
 * same or a smaller size allocate nothing.  RH_BF16: one image's activations at the network's
 * highest internal resolution must stay below 2 GiB (RH_E_SHAPE otherwise).
 */
rh_status rh_enhance(rh_ctx* ctx, const uint8_t* in, int32_t N, int32_t H, int32_t W,
                     float* out, const uint32_t* n_valid);

/*
 * Exact-border variant of rh_enhance for packed bins (in: dev u8 [N][S][S][3], S = bin_size).
 * rh_enhance pads every layer with zeros at the *bin* border only, so a box whose halo leaves the
 * frame carries non-zero activations where a whole-frame run has padding, and macroblocks within
 * the receptive field of a frame border differ from the frame-based result.  Here, after every
 * layer but the last, the activations of every placed box are set to zero where the box's source
 * pixels lie outside the frame (at that layer's resolution): with halo >= the network's
 * receptive-field radius the packed result then equals the frame-based one at every selected
 * macroblock, border ones included.  boxes / counts: dev, as written by rh_pack for these bins
 * (turned boxes are handled).  Costs one small extra launch per layer.
 */
rh_status rh_enhance_exact(rh_ctx* ctx, const uint8_t* in, int32_t N, const rh_box* boxes,
                           const uint32_t* counts, float* out, const uint32_t* n_valid);

/*
 * Box-masked variant of rh_enhance for packed bins (in: dev u8 [N][S][S][3], S = bin_size), for
 * RH_BF16 networks with 64 channels.  A packed bin is only partly occupied (Sec. 3.3.2, occupy
 * ratio), and the area no box covers is never pasted.  The bin is cut into cells of RH_CELL_H x
 * RH_CELL_W pixels from its origin; a cell is live when a placed box (with its halo; a turned box
 * with its exchanged extent) shares a pixel with it.  The output of the first conv and of every
 * conv of the body (after its residual / long-skip addition) is zero outside the live cells, and
 * the body's convs do not compute the other cells at all; the layers after the body (upsampling
 * convs, pixel shuffles, last conv) run on that tensor everywhere, so every output pixel is
 * written.  The result differs from rh_enhance's within the network's receptive field of a cell
 * that is not live (there the plain mode sees the activations of an empty area instead of zeros).
 * boxes / counts: dev, as written by rh_pack for these bins; N <= max_bins.  Costs three small
 * extra launches.  RH_E_UNIMPLEMENTED for other networks.
 */
#define RH_CELL_H 8
#define RH_CELL_W 32
rh_status rh_enhance_masked(rh_ctx* ctx, const uint8_t* in, int32_t N, const rh_box* boxes,
                            const uint32_t* counts, float* out, const uint32_t* n_valid);

/*
 * Needed-region variant of rh_enhance for packed bins (in: dev u8 [N][S][S][3]), for RH_BF16 networks
 * with 64 channels.  Only the pixels of placed macroblocks are pasted (Sec. 3.3.3), and a conv
 * output is read by the next conv within one pixel, so the part of a bin that can reach a pasted
 * pixel shrinks from layer to layer.  Every layer computes only the RH_CELL_H x RH_CELL_W cells
 * within its own radius (rh_needed_radii) of a placed macroblock.  On the pixels of the placed
 * macroblocks - what rh_unpack reads - the output is bit-identical to rh_enhance's; everywhere else
 * it is unspecified (not written, or computed from values that were not).  places / counts: dev,
 * as written by rh_pack for these bins (counts[3] = number of placement rows); N <= max_bins.
 * Costs two small extra launches; the first call allocates the mode's scratch.
 * RH_E_UNIMPLEMENTED for other networks and with per_layer_tail.
 */
rh_status rh_enhance_needed(rh_ctx* ctx, const uint8_t* in, int32_t N, const rh_mbplace* places,
                            const uint32_t* counts, float* out, const uint32_t* n_valid);

/*
 * Host only.  The radius, in low-resolution pixels (Chebyshev distance to the nearest pasted pixel),
 * within which each layer's output must be right for the pasted pixels to be: radii[0] the first
 * conv, radii[1 .. nb] the nb convs after it in execution order, radii[nb + 1] = 0 the layers
 * after the body.  Returns nb, or -1 when the mode does not cover the network or cap < nb + 2.
 */
int32_t rh_needed_radii(const rh_net_desc* net, int32_t per_layer_tail, int32_t* radii, int32_t cap);

/*
 * Paste (Sec. 3.3.3; problem statement of Sec. 3.2.1: SR on selected MBs, bilinear IN(.)
 * elsewhere).  frames_hr u8 [F][s*H][s*W][3] = bilinear interpolation of frames_lr (integer
 * factor s, half-pixel centres, edge clamp, exact integer arithmetic, round half up); every
 * placed MB's (16s x 16s) block is replaced by q = floor(255*e + 0.5),
 * e = clamp(base/255 + net, 0, 1) in fp32, net read from image `bin` of `enhanced`
 * (f32 [n_img][s*ih][s*iw][3]) at (s*px, s*py), transposed back if the place is turned.
 * Places with bin = 0xFFFF stay bilinear.  Of a block cut by the frame's right / bottom edge
 * (frame sides that are not multiples of 16) only the part inside the frame is pasted and sel
 * reports 0 for the rest.  A place is honoured when the in-frame part of its block lies inside
 * the enhanced image (whole MBs: px + 16 <= iw, py + 16 <= ih); otherwise the MB stays bilinear.
 * places/n_places: dev, from rh_pack (n_places = &counts[3]) or rh_identity_places; rows in ascending
 * mb_id (as both write them): the kernel finds a macroblock's row by searching.
 * sel (dev, may be NULL): f32 [n_places][16s][16s][3], the unquantised e of every placed MB.
 */
rh_status rh_unpack(rh_ctx* ctx, const float* enhanced, int32_t n_img, int32_t ih, int32_t iw,
                    const rh_mbplace* places, const uint32_t* n_places,
                    const uint8_t* frames_lr, int32_t F, uint8_t* frames_hr, float* sel);

/* Placement rows of the frame-based run: every MB selected, image f = frame f, px = 16*mbx.
 * places capacity F*MBH*MBW; n_places u32[1] (both dev). */
rh_status rh_identity_places(rh_ctx* ctx, int32_t F, rh_mbplace* places, uint32_t* n_places);

/* Synchronise the stream and copy counts (dev u32[4], as written by rh_pack) to the host.
 * Returns RH_E_CAPACITY if the overflow flag is set. */
rh_status rh_read_counts(rh_ctx* ctx, const uint32_t* counts, uint32_t out[4]);

/*
 * Temporal importance reuse (Sec. 3.2.2): predict the importance map only on the frames of a chunk
 * where a cheap feature of the codec's luma residual changes most, and let the other frames reuse
 * the map of such a frame.  Three calls, all asynchronous on the context's stream.
 *
 * rh_temporal_phi: the inverse-area operator Phi of every frame.  The paper names the operator and
 * what it reacts to (small changed objects) without a formula; as built: a pixel has changed when
 * |residual| > tau, blobs are the 8-connected sets of changed pixels of one frame, and
 * Phi = sum over blobs of at least min_area pixels of 1/area, kept exactly as the integer
 * sum of floor(2^32 / area) (order-independent, so the frame choice below is reproducible).
 *   res_y (dev): int16 [F][frame_h][frame_w], the Y residual of each frame, F <= max_frames of
 *   the context.  tau >= 0, min_area >= 1.  phi (dev out): uint64 [F].
 * Uses the context's workspace (16 bytes per pixel; grows like rh_enhance's); F*frame_h*frame_w must
 * stay below 2^31 (RH_E_SHAPE).
 */
rh_status rh_temporal_phi(rh_ctx* ctx, const int16_t* res_y, int32_t F, int32_t tau, int32_t min_area,
                          uint64_t* phi);

/*
 * rh_temporal_select: the frame choice.  stream_off (host): int32 [n_streams + 1], ascending,
 * stream s owns frames [stream_off[s], stream_off[s+1]) of the batch (at least 1, at most 2048
 * frames each; stream_off[0] = 0, stream_off[n_streams] = F; n_streams <= 1024).  Per stream, with
 * S_i = |Phi_{i+1} - Phi_i| L1-normalised over the chunk, frame f sits at position
 * P_f = S_0 + ... + S_{f-1} of the cumulative distribution (all 0 when nothing changed); [0,1] is
 * cut into N_s equal intervals, frame f lies in interval min(N_s - 1, floor(N_s * P_f)), and in
 * every interval that holds a frame the frame nearest the interval's midpoint (the earliest of
 * equally near ones) is predicted while the others reuse it.  The budget n_total (frames to
 * predict over all streams, n_streams <= n_total <= 65535) is shared out as one frame per stream
 * plus the rest in proportion to the streams' total change sum_i S_i before normalisation
 * (largest remainders, ties to the lower stream, equal shares if nothing changed anywhere).
 * All comparisons are exact integer arithmetic; F * (frame_h/2 + 1) * (frame_w/2 + 1) must stay
 * below 2^31 so that no sum of changes can pass 2^63 (RH_E_SHAPE otherwise).
 *   phi (dev): uint64 [F] as written by rh_temporal_phi.
 *   alloc (dev out): uint32 [n_streams], N_s.   selected (dev out): u8 [F], 1 = predict this frame.
 *   reuse_from (dev out): uint32 [F], the batch-wide index of the frame whose map frame f uses
 *   (itself for a predicted frame; never a frame of another stream).
 *   n_selected (dev out): uint32 [1], number of frames to predict (<= n_total: an interval that
 *   holds no frame selects nothing).
 */
rh_status rh_temporal_select(rh_ctx* ctx, const uint64_t* phi, const int32_t* stream_off, int32_t n_streams,
                             int32_t n_total, uint32_t* alloc, uint8_t* selected, uint32_t* reuse_from,
                             uint32_t* n_selected);

/*
 * rh_temporal_spread: the reuse itself.  importance (dev, in/out): f32 [F][MBH][MBW] holding valid
 * maps at the predicted frames; every other frame f receives a copy of frame reuse_from[f]'s map.
 * The result is what rh_select_regions takes.  selected / reuse_from as written by
 * rh_temporal_select (entries that point outside [0, F) or at a frame that is not predicted leave
 * frame f untouched).
 */
rh_status rh_temporal_spread(rh_ctx* ctx, float* importance, int32_t F, const uint8_t* selected,
                             const uint32_t* reuse_from);

/*
 * Measurement aid (not part of the method): when enabled, the kernel launches of the
 * calls above are bracketed by HIP events on the context's stream, one event pair around each run of
 * consecutive launches of a class (no event is placed between back-to-back launches).
 * rh_profile_read synchronises, adds up the elapsed times and launch counts since the last
 * read into ms[RH_PROF_N] / launches[RH_PROF_N] (host arrays) and resets them.
 * RH_PROF_CONV is the bf16 MFMA conv with C input and bf16 output channels (the body and the
 * upsampling convs), the kernel that dominates the path; with RH_FP32 it covers all layers.
 */
enum { RH_PROF_SELECT = 0, RH_PROF_PLAN = 1, RH_PROF_GATHER = 2, RH_PROF_HEAD = 3, RH_PROF_CONV = 4,
       RH_PROF_CONV_LAST = 5, RH_PROF_UNPACK = 6, RH_PROF_TEMPORAL = 7, RH_PROF_N = 8 };
rh_status rh_profile_enable(rh_ctx* ctx, int32_t on);
rh_status rh_profile_read(rh_ctx* ctx, double* ms, uint32_t* launches);

#ifdef __cplusplus
}
#endif
#endif /* RH_H */

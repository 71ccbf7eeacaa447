/*
 * CPU oracle for the region-aware enhancer (RegenHance, arXiv 2407.16990, Sec. 3.3).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain reference that the
 * HIP path is checked against.  It shares no code, header, table or helper with
 * the GPU library and must never be called from a product path: only tests,
 * the smoke check and the bench's cpu_baseline leg may use it.
 *
 * Everything is written as the plain definition (selection, gather, 3x3
 * convolution, pixel shuffle, bilinear interpolation, paste) or, for the
 * bin-packing heuristic, as the steps of Alg. 1 in the paper's order.  Loops
 * are naive; the only parallelism is OpenMP over independent images or, when a batch has fewer
 * images than there are threads, over the independent output rows of a convolution.
 * Floating point is fp64 except where a value decides an integer that the
 * GPU decides in fp32 (the box sort key's numerator and the final 8-bit
 * quantisation), which is done in fp32 here too.
 *
 * Pins (tests/test_oracle_*.py): brute-force packers/validators, flood fill,
 * exact rationals, delta-kernel convs, library conv/pixel-shuffle/bilinear as
 * second opinions, and a hand-traced placement example.  The plan produced by
 * the packing heuristic has no printed example in the paper: plan equality is
 * "parity unpinned" with respect to the paper and pinned only to the
 * determinism rules stated at orc_plan (tie-breaks, list order, split of the free remainder).
 *
 * The inverse-area operator of the temporal importance reuse (Sec. 3.2.2, orc_phi at the end of
 * the file) is pinned by hand cases and a library labelling routine
 * (tests/test_oracle_temporal.py); its formula is a reading of the paper, which prints none:
 * "parity unpinned" with respect to the paper.
 */
#include <math.h>
#include <omp.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define MBS 16 /* macroblock side in pixels (Sec. 3.2.1) */

/* ------------------------------------------------------------------------ */
/* Sec. 3.3.1, the N budget: the largest N with MB_size * N <= H * W * B.    */
long orc_budget(int bin_h, int bin_w, int n_bins)
{
    return ((long)bin_h * bin_w * n_bins) / (MBS * MBS);
}

/* ------------------------------------------------------------------------ */
/* Sec. 3.3.1 cross-stream MB selection.
 *
 * The global queue orders macroblocks by importance, highest first.  Reading
 * for what the paper leaves open: equal importance -> lower flat index first;
 * -0 equals +0; NaN ranks below every number.  Flat index g = (f*mbh+y)*mbw+x.
 */
typedef struct { float v; uint32_t g; } qent;

static int imp_rank_cmp(float a, float b) /* <0 if a ranks before (is more important than) b */
{
    int an = isnan(a), bn = isnan(b);
    if (an || bn) return an - bn;          /* NaN after numbers; two NaNs tie */
    if (a > b) return -1;
    if (a < b) return 1;
    return 0;                              /* includes -0 == +0 */
}

static int qent_cmp(const void* pa, const void* pb)
{
    const qent* a = (const qent*)pa; const qent* b = (const qent*)pb;
    int c = imp_rank_cmp(a->v, b->v);
    if (c) return c;
    return (a->g > b->g) - (a->g < b->g);
}

/* mode 0: top-k per segment; mode 1: importance >= thr per segment.
 * segs[i] = {frame_begin, frame_end, k}; thr[i] used in mode 1.
 * Outputs: mask[F*mbh*mbw] (0/1), list (ascending g), *n_sel.  Returns 0, or
 * -1 for malformed segments (out of range, overlapping or unordered). */
int orc_select(const float* imp, int F, int mbh, int mbw,
               const uint32_t* segs, const float* thr, int nseg, int mode,
               uint8_t* mask, uint32_t* list, uint32_t* n_sel)
{
    size_t per = (size_t)mbh * mbw, total = per * F;
    memset(mask, 0, total);
    uint32_t prev_end = 0;
    for (int s = 0; s < nseg; ++s) {
        uint32_t fb = segs[3 * s], fe = segs[3 * s + 1], k = segs[3 * s + 2];
        if (fb > fe || fe > (uint32_t)F || fb < prev_end) return -1;
        prev_end = fe;
        size_t n = (size_t)(fe - fb) * per, g0 = (size_t)fb * per;
        if (mode == 1) {
            for (size_t i = 0; i < n; ++i)
                if (imp[g0 + i] >= thr[s]) mask[g0 + i] = 1;   /* NaN compares false */
            continue;
        }
        qent* q = (qent*)malloc((n ? n : 1) * sizeof(qent));
        for (size_t i = 0; i < n; ++i) { q[i].v = imp[g0 + i]; q[i].g = (uint32_t)(g0 + i); }
        qsort(q, n, sizeof(qent), qent_cmp);
        if (k > n) k = (uint32_t)n;
        for (uint32_t i = 0; i < k; ++i) mask[q[i].g] = 1;
        free(q);
    }
    uint32_t c = 0;
    for (size_t g = 0; g < total; ++g) if (mask[g]) list[c++] = (uint32_t)g;
    *n_sel = c;
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Alg. 1: region-aware bin packing, on macroblock indexes only.             */

typedef struct {
    int frame, mbx0, mby0, wmb, hmb;
    int id;          /* smallest flat index among the MBs the box owns */
    float sum;       /* fp32 sum of owned importance, ascending flat index */
    double key;      /* sort key, larger first: importance density = sum / (wmb*hmb), or the area */
    int bin, bx, by;
    int rot;         /* 1: packed turned (rows and columns exchanged) */
} obox;

typedef struct { int bin, x, y, w, h; } orect;

static int imin(int a, int b) { return a < b ? a : b; }
static int imax(int a, int b) { return a > b ? a : b; }

static int obox_cmp(const void* pa, const void* pb)
{
    const obox* a = (const obox*)pa; const obox* b = (const obox*)pb;
    int an = isnan(a->key), bn = isnan(b->key);
    if (an != bn) return an - bn;                              /* NaN density ranks last */
    if (!an) {
        if (a->key > b->key) return -1;   /* higher density first (Alg. 1, Sort) */
        if (a->key < b->key) return 1;
    }
    return (a->id > b->id) - (a->id < b->id);
}

/* Output rows: boxes_out[i] = {frame, mbx0, mby0, wmb, hmb, rot, bin, bx, by, id}
 *              places_out[j] = {mb_id, box, bin, px, py}  (ascending mb_id)
 *              place_rot_out[j] (may be NULL) = rot of the MB's box
 * counts_out = {n_boxes, n_bins, overflow}.
 * sort_policy 0: importance density first (Alg. 1, Sort); 1: the classic large-item-first
 * order the paper compares against (box area in MBs, descending).  Ties: ascending box id.
 * rotate 0: boxes keep their orientation.  1: RotatePacking of Alg. 1 - a free area also
 * accepts the box turned by a quarter, here read as "rows and columns exchanged"; the box is
 * kept upright when it fits upright.  A turned box occupies (bh x bw) pixels; the MB at
 * offset (dx, dy) of the upright box starts at (bx + dy, by + dx) and its pixels are
 * transposed.
 * On overflow (more than max_bins bins needed) the first box that cannot be
 * placed and every later one get bin = 0xFFFF, bx = by = 0 (their MBs px = py = 0).
 * conn: 4 or 8.  T: largest box side in MBs (the partition's preset size).
 * Returns 0, or -1 on invalid geometry. */
int orc_plan(const uint8_t* mask, const float* imp, int F, int mbh, int mbw,
             int halo, int bin_size, int conn, int T, int max_bins, int sort_policy, int rotate,
             int32_t* boxes_out, int32_t* places_out, int32_t* place_rot_out, int32_t* counts_out)
{
    int per = mbh * mbw, total = per * F;
    if (F < 0 || mbh < 1 || mbw < 1) return -1;
    size_t tn = (size_t)(total ? total : 1);
    int minside = MBS + 2 * halo;
    if (T < 1 || MBS * T + 2 * halo > bin_size || (conn != 4 && conn != 8)) return -1;

    /* RegionProps: connected components of selected MBs inside each frame. */
    int* comp = (int*)malloc(sizeof(int) * tn);
    int* stack = (int*)malloc(sizeof(int) * (per ? per : 1));
    for (int g = 0; g < total; ++g) comp[g] = -1;
    int ncomp = 0;
    int* comp_first = (int*)malloc(sizeof(int) * tn);
    for (int g = 0; g < total; ++g) {
        if (!mask[g] || comp[g] >= 0) continue;
        int f = g / per;
        comp_first[ncomp] = g;
        int sp = 0; stack[sp++] = g; comp[g] = ncomp;
        while (sp) {
            int c = stack[--sp];
            int cy = (c % per) / mbw, cx = c % mbw;
            for (int dy = -1; dy <= 1; ++dy) for (int dx = -1; dx <= 1; ++dx) {
                if (!dy && !dx) continue;
                if (conn == 4 && dy && dx) continue;
                int ny = cy + dy, nx = cx + dx;
                if (ny < 0 || ny >= mbh || nx < 0 || nx >= mbw) continue;
                int n = f * per + ny * mbw + nx;
                if (mask[n] && comp[n] < 0) { comp[n] = ncomp; stack[sp++] = n; }
            }
        }
        ++ncomp;
    }

    /* Bound: bounding box of each region, in MB units. */
    int* bx0 = (int*)malloc(sizeof(int) * (ncomp + 1)); int* bx1 = (int*)malloc(sizeof(int) * (ncomp + 1));
    int* by0 = (int*)malloc(sizeof(int) * (ncomp + 1)); int* by1 = (int*)malloc(sizeof(int) * (ncomp + 1));
    for (int c = 0; c < ncomp; ++c) { bx0[c] = by0[c] = 1 << 30; bx1[c] = by1[c] = -1; }
    for (int g = 0; g < total; ++g) {
        int c = comp[g]; if (c < 0) continue;
        int y = (g % per) / mbw, x = g % mbw;
        bx0[c] = imin(bx0[c], x); bx1[c] = imax(bx1[c], x);
        by0[c] = imin(by0[c], y); by1[c] = imax(by1[c], y);
    }

    /* Partition: cut boxes larger than T on a T x T grid anchored at the box's
     * top-left; each cell shrinks to the bounding box of the region's own MBs
     * inside it; empty cells vanish.  A box owns exactly those MBs. */
    obox* boxes = (obox*)malloc(sizeof(obox) * tn);
    int* owner_id = (int*)malloc(sizeof(int) * tn);   /* id of the owning box */
    for (int g = 0; g < total; ++g) owner_id[g] = -1;
    int nb = 0;
    for (int c = 0; c < ncomp; ++c) {
        int f = comp_first[c] / per;
        for (int cy = by0[c]; cy <= by1[c]; cy += T) for (int cx = bx0[c]; cx <= bx1[c]; cx += T) {
            int x0 = 1 << 30, y0 = 1 << 30, x1 = -1, y1 = -1, id = -1; float sum = 0.0f;
            for (int y = cy; y < cy + T && y <= by1[c]; ++y) for (int x = cx; x < cx + T && x <= bx1[c]; ++x) {
                int g = f * per + y * mbw + x;
                if (comp[g] != c) continue;
                if (id < 0) id = g;
                owner_id[g] = id;
                sum = sum + imp[g];             /* fp32, ascending flat index */
                x0 = imin(x0, x); x1 = imax(x1, x);
                y0 = imin(y0, y); y1 = imax(y1, y);
            }
            if (id < 0) continue;
            obox* b = &boxes[nb++];
            b->frame = f; b->mbx0 = x0; b->mby0 = y0; b->wmb = x1 - x0 + 1; b->hmb = y1 - y0 + 1;
            b->id = id; b->sum = sum;
            b->key = sort_policy == 1 ? (double)(b->wmb * b->hmb) : (double)sum / (double)(b->wmb * b->hmb);
            b->bin = -1; b->bx = b->by = 0; b->rot = 0;
        }
    }

    /* Sort by importance density, highest first; ties by box id. */
    qsort(boxes, nb, sizeof(obox), obox_cmp);
    int* idx_of_id = (int*)malloc(sizeof(int) * tn);  /* box id -> sorted position */
    for (int i = 0; i < nb; ++i) idx_of_id[boxes[i].id] = i;

    /* First-fit over the ordered free-area list.  Bins are opened on demand
     * (the list starts empty); a new bin's whole area joins the tail. */
    int cap = 2 * nb + 4, nfree = 0, nbins = 0, overflow = 0;
    orect* fr = (orect*)malloc(sizeof(orect) * cap);
    for (int i = 0; i < nb; ++i) {
        obox* b = &boxes[i];
        int bw = MBS * b->wmb + 2 * halo, bh = MBS * b->hmb + 2 * halo;
        if (overflow) { b->bin = 0xFFFF; continue; }
        int at = -1;
        for (int j = 0; j < nfree; ++j) {
            int upright = fr[j].w >= bw && fr[j].h >= bh;
            int turned = rotate && fr[j].w >= bh && fr[j].h >= bw;      /* RotatePacking */
            if (upright || turned) { at = j; b->rot = !upright; break; }
        }
        if (b->rot) { int t = bw; bw = bh; bh = t; }                    /* occupied size */
        if (at < 0) {
            if (nbins >= max_bins) { overflow = 1; b->bin = 0xFFFF; continue; }
            fr[nfree].bin = nbins++; fr[nfree].x = 0; fr[nfree].y = 0;
            fr[nfree].w = bin_size; fr[nfree].h = bin_size;
            at = nfree++;
        }
        orect fa = fr[at];
        b->bin = fa.bin; b->bx = fa.x; b->by = fa.y;      /* top-left of the free area */
        /* Update: the L-shaped remainder is split into its largest rectangle
         * plus the rest (reading of InnerFree, Appx. A). */
        long ar = (long)(fa.w - bw) * fa.h, ab = (long)fa.w * (fa.h - bh);
        orect right = { fa.bin, fa.x + bw, fa.y, fa.w - bw, 0 };
        orect bottom = { fa.bin, fa.x, fa.y + bh, 0, fa.h - bh };
        if (ar >= ab) { right.h = fa.h; bottom.w = bw; }
        else          { right.h = bh;   bottom.w = fa.w; }
        int keep_r = right.w >= minside && right.h >= minside;
        int keep_b = bottom.w >= minside && bottom.h >= minside;
        orect ins[2]; int ni = 0;
        if (keep_r && keep_b) {
            long a_r = (long)right.w * right.h, a_b = (long)bottom.w * bottom.h;
            if (a_b < a_r) { ins[0] = bottom; ins[1] = right; }
            else           { ins[0] = right;  ins[1] = bottom; }   /* smaller first; tie: right first */
            ni = 2;
        } else if (keep_r) { ins[0] = right; ni = 1; }
        else if (keep_b)   { ins[0] = bottom; ni = 1; }
        /* replace fr[at] by ins[0..ni) in place, keeping list order */
        int delta = ni - 1;
        if (delta > 0) for (int j = nfree - 1; j > at; --j) fr[j + delta] = fr[j];
        if (delta < 0) for (int j = at + 1; j < nfree; ++j) fr[j + delta] = fr[j];
        for (int j = 0; j < ni; ++j) fr[at + j] = ins[j];
        nfree += delta;
    }

    for (int i = 0; i < nb; ++i) {
        int32_t* o = boxes_out + 10 * i; obox* b = &boxes[i];
        o[0] = b->frame; o[1] = b->mbx0; o[2] = b->mby0; o[3] = b->wmb; o[4] = b->hmb;
        o[5] = b->rot; o[6] = b->bin; o[7] = b->bx; o[8] = b->by; o[9] = b->id;
    }
    /* Placement of every selected MB, ascending flat index. */
    int np = 0;
    for (int g = 0; g < total; ++g) {
        if (!mask[g]) continue;
        int y = (g % per) / mbw, x = g % mbw, found = idx_of_id[owner_id[g]];
        obox* b = &boxes[found];
        int dx = halo + MBS * (x - b->mbx0), dy = halo + MBS * (y - b->mby0);
        if (place_rot_out) place_rot_out[np] = b->rot;
        int32_t* o = places_out + 5 * np++;
        o[0] = g; o[1] = found; o[2] = b->bin;
        o[3] = b->bin == 0xFFFF ? 0 : b->bx + (b->rot ? dy : dx);
        o[4] = b->bin == 0xFFFF ? 0 : b->by + (b->rot ? dx : dy);
    }
    counts_out[0] = nb; counts_out[1] = nbins; counts_out[2] = overflow;
    free(comp); free(stack); free(comp_first); free(bx0); free(bx1); free(by0); free(by1);
    free(boxes); free(owner_id); free(idx_of_id); free(fr);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Sec. 3.3.3: stitch real pixels into the bins following the plan.
 * bins[b][y][x][c] is zero everywhere except inside placed boxes, where it is
 * the frame pixel under the box (zero where the box's halo leaves the frame).
 * A turned box (rot = 1) is stored with rows and columns exchanged. */
void orc_gather(const uint8_t* frames, int F, int H, int W,
                const int32_t* boxes, int n_boxes, int halo, int bin_size, int n_bins,
                uint8_t* bins)
{
    (void)F;
    size_t S = (size_t)bin_size;
    memset(bins, 0, (size_t)n_bins * S * S * 3);
    for (int i = 0; i < n_boxes; ++i) {
        const int32_t* b = boxes + 10 * i;
        int f = b[0], bin = b[6];
        if (bin < 0 || bin >= n_bins) continue;
        int bw = MBS * b[3] + 2 * halo, bh = MBS * b[4] + 2 * halo;
        int sx0 = MBS * b[1] - halo, sy0 = MBS * b[2] - halo;
        for (int j = 0; j < bh; ++j) for (int k = 0; k < bw; ++k) {
            int sy = sy0 + j, sx = sx0 + k;
            for (int c = 0; c < 3; ++c) {
                uint8_t v = 0;
                if (sy >= 0 && sy < H && sx >= 0 && sx < W)
                    v = frames[(((size_t)f * H + sy) * W + sx) * 3 + c];
                int row = b[5] ? k : j, col = b[5] ? j : k;
                bins[(((size_t)bin * S + (b[8] + row)) * S + (b[7] + col)) * 3 + c] = v;
            }
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Bilinear interpolation IN(.) of the problem statement (Sec. 3.2.1), integer
 * factor s, half-pixel centres, edge clamp.  All weights are multiples of
 * 1/(2s), so the result is computed exactly in integers, rounding half up. */
void orc_bilinear(const uint8_t* in, int H, int W, int s, uint8_t* out)
{
    int D = 2 * s, HH = H * s, WW = W * s;
    for (int Y = 0; Y < HH; ++Y) {
        int ny = 2 * Y + 1 - s;
        int y0 = (ny >= 0) ? ny / D : -1;
        int wy1 = ny - y0 * D, wy0 = D - wy1;
        int ya = y0 < 0 ? 0 : y0, yb = y0 + 1 > H - 1 ? H - 1 : y0 + 1;
        for (int X = 0; X < WW; ++X) {
            int nx = 2 * X + 1 - s;
            int x0 = (nx >= 0) ? nx / D : -1;
            int wx1 = nx - x0 * D, wx0 = D - wx1;
            int xa = x0 < 0 ? 0 : x0, xb = x0 + 1 > W - 1 ? W - 1 : x0 + 1;
            for (int c = 0; c < 3; ++c) {
                int p00 = in[((size_t)ya * W + xa) * 3 + c], p01 = in[((size_t)ya * W + xb) * 3 + c];
                int p10 = in[((size_t)yb * W + xa) * 3 + c], p11 = in[((size_t)yb * W + xb) * 3 + c];
                int acc = wy0 * (wx0 * p00 + wx1 * p01) + wy1 * (wx0 * p10 + wx1 * p11);
                out[((size_t)Y * WW + X) * 3 + c] = (uint8_t)((acc + D * D / 2) / (D * D));
            }
        }
    }
}

/* ------------------------------------------------------------------------ */
/* SR model (Sec. 3.3.3): plain definitions of its layers, channels-last.    */

/* out[y][x][co] = b[co] + sum_{ky,kx,ci} w[co][ky][kx][ci] * in[y+ky-1][x+kx-1][ci],
 * zero outside the tensor; optional ReLU. */
void orc_conv3x3(const double* in, int H, int W, int Cin, const float* w, const float* b,
                 int Cout, int relu, double* out)
{
    /* every output value is computed on its own: rows may go to different threads (this pragma is
     * inert inside orc_sr_forward's parallel loop over images, nested parallelism being off) */
#pragma omp parallel for schedule(dynamic, 1)
    for (int y = 0; y < H; ++y) for (int x = 0; x < W; ++x) for (int co = 0; co < Cout; ++co) {
        double acc = (double)b[co];
        for (int ky = 0; ky < 3; ++ky) {
            int yy = y + ky - 1; if (yy < 0 || yy >= H) continue;
            for (int kx = 0; kx < 3; ++kx) {
                int xx = x + kx - 1; if (xx < 0 || xx >= W) continue;
                const double* ip = in + ((size_t)yy * W + xx) * Cin;
                const float* wp = w + (((size_t)co * 3 + ky) * 3 + kx) * Cin;
                for (int ci = 0; ci < Cin; ++ci) acc += (double)wp[ci] * ip[ci];
            }
        }
        if (relu && acc < 0.0) acc = 0.0;
        out[((size_t)y * W + x) * Cout + co] = acc;
    }
}

/* out[y*r+i][x*r+j][c] = in[y][x][c*r*r + i*r + j] */
void orc_pixel_shuffle(const double* in, int H, int W, int C, int r, double* out)
{
    int Co = C / (r * r);
    for (int y = 0; y < H; ++y) for (int x = 0; x < W; ++x)
        for (int c = 0; c < Co; ++c) for (int i = 0; i < r; ++i) for (int j = 0; j < r; ++j)
            out[(((size_t)(y * r + i)) * (W * r) + (x * r + j)) * Co + c] =
                in[((size_t)y * W + x) * C + c * r * r + i * r + j];
}

typedef struct { const float* w; const float* b; } olayer;

static const float* take_layer(const float** p, int cin, int cout, olayer* L)
{
    L->w = *p; L->b = *p + (size_t)cout * 9 * cin; *p = L->b + cout; return L->w;
}

static double* dalloc(size_t n) { return (double*)malloc(sizeof(double) * (n ? n : 1)); }

/* Exact-border mode: keep (u8 [H][W], may be NULL) is 0 at the pixels of the image that lie
 * outside the source frame (halo of a box that leaves the frame).  Every layer's output is set
 * to zero there, at that layer's resolution (rr x the input's), so that the next convolution
 * sees what per-layer zero padding at the frame border gives in a whole-frame run. */
static void apply_keep(double* buf, int h, int w, int C, const uint8_t* keep, int rr)
{
    if (!keep) return;
    int W0 = w / rr;
    for (int y = 0; y < h; ++y) for (int x = 0; x < w; ++x)
        if (!keep[(size_t)(y / rr) * W0 + x / rr])
            for (int c = 0; c < C; ++c) buf[((size_t)y * w + x) * C + c] = 0.0;
}

/* One image through the network.  topology: 0 plain, 1 res, 2 edsr.
 * in: u8 [H][W][3]; out: fp64 [sH][sW][3] (the network's raw output). */
static void sr_one(int topology, int C, int nblk, int s, const float* blob,
                   const uint8_t* in, int H, int W, const uint8_t* keep, int keep_tail, double* out)
{
    size_t px = (size_t)H * W;
    const float* p = blob; olayer L;
    double* x = dalloc(px * 3);
    for (size_t i = 0; i < px * 3; ++i) x[i] = (double)in[i] / 255.0;
    double* a = dalloc(px * C); double* t = dalloc(px * C);
    if (topology == 0) {
        take_layer(&p, 3, C, &L); orc_conv3x3(x, H, W, 3, L.w, L.b, C, 1, a);
        apply_keep(a, H, W, C, keep, 1);
        for (int l = 0; l < nblk - 2; ++l) {
            take_layer(&p, C, C, &L); orc_conv3x3(a, H, W, C, L.w, L.b, C, 1, t);
            apply_keep(t, H, W, C, keep, 1);
            double* sw = a; a = t; t = sw;
        }
        int Co = 3 * s * s; double* y = dalloc(px * Co);
        take_layer(&p, C, Co, &L); orc_conv3x3(a, H, W, C, L.w, L.b, Co, 0, y);
        orc_pixel_shuffle(y, H, W, Co, s, out); free(y);
    } else {
        take_layer(&p, 3, C, &L); orc_conv3x3(x, H, W, 3, L.w, L.b, C, 0, a);
        apply_keep(a, H, W, C, keep, 1);
        double* head = NULL;
        if (topology == 2) { head = dalloc(px * C); memcpy(head, a, sizeof(double) * px * C); }
        double* u = dalloc(px * C);
        for (int blk = 0; blk < nblk; ++blk) {          /* x <- x + conv(relu(conv(x))) */
            take_layer(&p, C, C, &L); orc_conv3x3(a, H, W, C, L.w, L.b, C, 1, t);
            apply_keep(t, H, W, C, keep, 1);
            take_layer(&p, C, C, &L); orc_conv3x3(t, H, W, C, L.w, L.b, C, 0, u);
            for (size_t i = 0; i < px * C; ++i) a[i] = a[i] + u[i];
            apply_keep(a, H, W, C, keep, 1);
        }
        if (topology == 1) {
            int Co = 3 * s * s; double* y = dalloc(px * Co);
            take_layer(&p, C, Co, &L); orc_conv3x3(a, H, W, C, L.w, L.b, Co, 0, y);
            orc_pixel_shuffle(y, H, W, Co, s, out); free(y);
        } else {
            take_layer(&p, C, C, &L); orc_conv3x3(a, H, W, C, L.w, L.b, C, 0, u);
            for (size_t i = 0; i < px * C; ++i) u[i] = u[i] + head[i];   /* long skip */
            apply_keep(u, H, W, C, keep, 1);
            int h = H, w = W; double* cur = u; u = NULL;
            int stages = (s == 4) ? 2 : 1, r = (s == 4) ? 2 : s;
            for (int st = 0; st < stages; ++st) {
                int Co = C * r * r; double* y = dalloc((size_t)h * w * Co);
                take_layer(&p, C, Co, &L); orc_conv3x3(cur, h, w, C, L.w, L.b, Co, 0, y);
                double* z = dalloc((size_t)h * w * Co);
                orc_pixel_shuffle(y, h, w, Co, r, z); free(y); free(cur);
                cur = z; h *= r; w *= r;
                if (keep_tail) apply_keep(cur, h, w, C, keep, h / H);
            }
            take_layer(&p, C, 3, &L); orc_conv3x3(cur, h, w, C, L.w, L.b, 3, 0, out);
            free(cur);
        }
        free(u); free(head);
    }
    free(x); free(a); free(t);
}

/* Batch of N images, each u8 [H][W][3] -> fp64 [sH][sW][3].  keep: NULL, or u8 [N][H][W] for the
 * exact-border mode (see apply_keep). */
void orc_sr_forward(int topology, int C, int nblk, int s, const float* blob,
                    const uint8_t* in, int N, int H, int W, const uint8_t* keep, double* out)
{
    size_t ipx = (size_t)H * W * 3, opx = ipx * s * s;
#pragma omp parallel for schedule(dynamic, 1) if (N >= omp_get_max_threads())
    for (int n = 0; n < N; ++n)
        sr_one(topology, C, nblk, s, blob, in + n * ipx, H, W, keep ? keep + (size_t)n * H * W : NULL, 1, out + n * opx);
}

/* Box-masked mode (Sec. 3.3.2: packed bins are only partly occupied; the area no box covers need
 * not be enhanced).  keep u8 [N][H][W] as written by orc_cell_keep.  The output of the first conv
 * and of every conv of the body (after its residual / long-skip addition) is set to zero where
 * keep == 0; the layers after the body - upsampling convs, pixel shuffles, last conv - run on
 * that tensor unmasked. */
void orc_sr_forward_masked(int topology, int C, int nblk, int s, const float* blob,
                           const uint8_t* in, int N, int H, int W, const uint8_t* keep, double* out)
{
    size_t ipx = (size_t)H * W * 3, opx = ipx * s * s;
#pragma omp parallel for schedule(dynamic, 1) if (N >= omp_get_max_threads())
    for (int n = 0; n < N; ++n)
        sr_one(topology, C, nblk, s, blob, in + n * ipx, H, W, keep + (size_t)n * H * W, 0, out + n * opx);
}

/* Box-masked mode: the bin is cut into cells of cell_h x cell_w pixels from its origin (cells at
 * the right / bottom edge may be cut).  keep[b][y][x] = 1 where the cell of pixel (x, y) shares
 * at least one pixel with a box placed in bin b (the box with its halo; a turned box occupies
 * its exchanged extent), 0 elsewhere. */
void orc_cell_keep(const int32_t* boxes, int n_boxes, int halo, int bin_size, int n_bins,
                   int cell_h, int cell_w, uint8_t* keep)
{
    size_t S = (size_t)bin_size;
    memset(keep, 0, (size_t)n_bins * S * S);
    for (int i = 0; i < n_boxes; ++i) {
        const int32_t* b = boxes + 10 * i;
        int bin = b[6];
        if (bin < 0 || bin >= n_bins) continue;
        int bw = MBS * b[3] + 2 * halo, bh = MBS * b[4] + 2 * halo;
        int fw = b[5] ? bh : bw, fh = b[5] ? bw : bh;            /* extent inside the bin */
        int cx0 = b[7] / cell_w, cx1 = (b[7] + fw - 1) / cell_w;
        int cy0 = b[8] / cell_h, cy1 = (b[8] + fh - 1) / cell_h;
        for (int y = cy0 * cell_h; y < (cy1 + 1) * cell_h && y < (int)S; ++y)
            for (int x = cx0 * cell_w; x < (cx1 + 1) * cell_w && x < (int)S; ++x)
                keep[((size_t)bin * S + y) * S + x] = 1;
    }
}

/* Exact-border mode: keep[b][y][x] = 0 where bin pixel (x, y) belongs to a placed box and its
 * source pixel lies outside the frame, 1 everywhere else. */
void orc_border_keep(int H, int W, const int32_t* boxes, int n_boxes, int halo, int bin_size, int n_bins,
                     uint8_t* keep)
{
    size_t S = (size_t)bin_size;
    memset(keep, 1, (size_t)n_bins * S * S);
    for (int i = 0; i < n_boxes; ++i) {
        const int32_t* b = boxes + 10 * i;
        int bin = b[6];
        if (bin < 0 || bin >= n_bins) continue;
        int bw = MBS * b[3] + 2 * halo, bh = MBS * b[4] + 2 * halo;
        int sx0 = MBS * b[1] - halo, sy0 = MBS * b[2] - halo;
        for (int j = 0; j < bh; ++j) for (int k = 0; k < bw; ++k) {
            int sy = sy0 + j, sx = sx0 + k;
            if (sy >= 0 && sy < H && sx >= 0 && sx < W) continue;
            int row = b[5] ? k : j, col = b[5] ? j : k;
            keep[((size_t)bin * S + (b[8] + row)) * S + (b[7] + col)] = 0;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Paste (Sec. 3.3.3; Eq. of Sec. 3.2.1: SR on selected MBs, IN elsewhere).
 * frames_hr = bilinear base everywhere; each placed MB's (16s x 16s) block is
 * replaced by clamp(base/255 + net_out, 0, 1) quantised to 8 bits.  The last
 * three operations are taken in fp32 because they decide an integer that the
 * GPU decides in fp32.  net: fp64 [n_img][s*ih][s*iw][3].  places rows and place_rot
 * (may be NULL = none turned) as in orc_plan.  sel (optional): fp32 [k][16s][16s][3], the
 * unquantised values.
 * H, W need not be multiples of 16: the macroblock grid is ceil(H/16) x ceil(W/16) and the part
 * of an edge macroblock that lies outside the frame is neither written nor reported (sel = 0).
 * A place is honoured when the in-frame part of its block lies inside the enhanced image (the
 * frame-based run's identity placement on such frames); otherwise the MB stays bilinear. */
void orc_unpack(const uint8_t* frames_lr, int F, int H, int W, int s,
                const double* net, int ih, int iw,
                const int32_t* places, const int32_t* place_rot, int k, int mbw_frame, int mbh_frame,
                uint8_t* frames_hr, float* sel)
{
    size_t lr = (size_t)H * W * 3, hr = lr * s * s;
#pragma omp parallel for schedule(dynamic, 1)
    for (int f = 0; f < F; ++f) orc_bilinear(frames_lr + f * lr, H, W, s, frames_hr + f * hr);
    int per = mbw_frame * mbh_frame, B = MBS * s, WW = W * s;
    size_t nimg = (size_t)ih * s * iw * s * 3;
    for (int i = 0; i < k; ++i) {
        const int32_t* pl = places + 5 * i;
        int g = pl[0], bin = pl[2], px = pl[3], py = pl[4];
        if (bin == 0xFFFF) continue;
        int f = g / per, my = (g % per) / mbw_frame, mx = g % mbw_frame;
        int fh = imin(B, H * s - my * B), fw = imin(B, WW - mx * B);           /* in-frame part */
        int rot = place_rot && place_rot[i];
        if (px * s + (rot ? fh : fw) > iw * s || py * s + (rot ? fw : fh) > ih * s) {
            if (sel) memset(sel + (size_t)i * B * B * 3, 0, sizeof(float) * B * B * 3);
            continue;
        }
        for (int y = 0; y < B; ++y) for (int x = 0; x < B; ++x) for (int c = 0; c < 3; ++c) {
            if (sel) sel[(((size_t)i * B + y) * B + x) * 3 + c] = 0.0f;
            if (my * B + y >= H * s || mx * B + x >= WW) continue;             /* outside the frame */
            size_t di = (size_t)f * hr + (((size_t)(my * B + y)) * WW + (mx * B + x)) * 3 + c;
            int ny = y, nx = x;
            if (place_rot && place_rot[i]) { ny = x; nx = y; }   /* turned box: transposed back */
            size_t si = (size_t)bin * nimg + (((size_t)(py * s + ny)) * (iw * s) + (px * s + nx)) * 3 + c;
            float base = (float)frames_hr[di] / 255.0f;
            float e = base + (float)net[si];
            e = e < 0.0f ? 0.0f : (e > 1.0f ? 1.0f : e);
            if (sel) sel[(((size_t)i * B + y) * B + x) * 3 + c] = e;
            float q = e * 255.0f;
            q = q + 0.5f;
            frames_hr[di] = (uint8_t)floorf(q);
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Temporal importance reuse (Sec. 3.2.2): the inverse-area operator Phi on the luma residual
 * of each frame.  The paper names the operator and what it responds to (small changed objects,
 * where the plain area feature responds to large ones) but prints no formula; the reading taken:
 *   1. a pixel has changed when |residual| > tau;
 *   2. blobs are the 8-connected components of the changed pixels of one frame (the same
 *      neighbourhood as the region labelling of Alg. 1);
 *   3. Phi = sum over blobs with area >= min_area of 1 / area.
 * Phi is kept as an integer in units of 2^-32, each term floor(2^32 / area): the frame choice
 * that follows compares sums of these values, and integer sums do not depend on the order the
 * blobs are met in.  res: int16 [F][H][W].  phi_q32: uint64 [F].  n_blobs (optional): int32 [F],
 * the number of blobs counted (after the min_area filter).
 * Plain flood fill with an explicit stack, one frame after the other. */
void orc_phi(const int16_t* res, int F, int H, int W, int tau, int min_area,
             uint64_t* phi_q32, int32_t* n_blobs)
{
    size_t per = (size_t)H * W;
    uint8_t* seen = (uint8_t*)malloc(per ? per : 1);
    int32_t* stack = (int32_t*)malloc(sizeof(int32_t) * (per ? per : 1));
    for (int f = 0; f < F; ++f) {
        const int16_t* r = res + f * per;
        memset(seen, 0, per);
        uint64_t phi = 0;
        int32_t nb = 0;
        for (int y0 = 0; y0 < H; ++y0) for (int x0 = 0; x0 < W; ++x0) {
            size_t p0 = (size_t)y0 * W + x0;
            if (seen[p0] || abs((int)r[p0]) <= tau) continue;
            int top = 0;
            long area = 0;
            stack[top++] = (int32_t)p0; seen[p0] = 1;
            while (top) {
                int32_t p = stack[--top];
                ++area;
                int y = p / W, x = p % W;
                for (int dy = -1; dy <= 1; ++dy) for (int dx = -1; dx <= 1; ++dx) {
                    int yy = y + dy, xx = x + dx;
                    if ((dy == 0 && dx == 0) || yy < 0 || yy >= H || xx < 0 || xx >= W) continue;
                    size_t q = (size_t)yy * W + xx;
                    if (seen[q] || abs((int)r[q]) <= tau) continue;
                    seen[q] = 1; stack[top++] = (int32_t)q;
                }
            }
            if (area >= min_area) { phi += ((uint64_t)1 << 32) / (uint64_t)area; ++nb; }
        }
        phi_q32[f] = phi;
        if (n_blobs) n_blobs[f] = nb;
    }
    free(seen); free(stack);
}

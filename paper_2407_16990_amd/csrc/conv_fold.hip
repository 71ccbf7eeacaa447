// The upsampler and the last conv of the EDSR-shaped nets as ONE convolution (Sec. 3.3.3: the
// enhancement model applied to the packed bins).
//
// After the body, these nets are linear: conv C -> C*r*r, pixel shuffle (once, or twice by 2 for
// x4), conv C -> 3, with no activation in between.  A composition of linear maps is a linear map:
// every output pixel (s*y + i, s*x + j) is a bias plus a weighted sum over the 5 x 5 neighbourhood
// of low-resolution pixel (y, x) of the body's output t,
//     out[s*y+i][s*x+j][co] = B[i][j][co] + sum_{dy,dx in -2..2} sum_ci Wc[i][j][co][dy][dx][ci] * t[y+dy][x+dx][ci],
// i.e. a 5 x 5 convolution C -> 3*s*s at low resolution followed by a pixel shuffle.  Executed
// that way the high-resolution 64-channel tensors (2.4 GB written and read back per batch at x4)
// never exist and the arithmetic shrinks about sevenfold.
//
// Wc and B are computed once at rh_create (in double, from the given weights) by pushing the
// gradient of each output through the layers, then rounded to bf16 for the matrix cores.  The
// layers pad with zeros at their own tensor's border, so the intermediate tensors outside the
// image are zero, not "what the previous conv would give there": Wc differs for the pixels of the
// outermost low-resolution ring.  There are 9 position classes (top / middle / bottom row x left
// / middle / right column); the main kernel computes every pixel with the middle class, a small
// second kernel recomputes the ring with the class weights.
//
// Main kernel: implicit GEMM on v_mfma_f32_32x32x16_bf16, D[row][pixel], rows = (i, j, co) of one
// 32-row chunk (x4: two chunks of two output rows i each; x2, x3: one chunk), N = 32 pixels of an
// image row, K = tap * C + ci over 25 taps.  One persistent 256-thread workgroup per CU keeps its
// chunk's weights (25 * C/16 KB) in LDS, stages a 12 x 36 pixel patch per 8 x 32 tile (same
// channels-last layout and XOR swizzle as the 3 x 3 kernels), and prefetches the next patch into
// registers during the MFMA loop.  A wave owns two pixel rows: per (kx, k-step) it reads 5 weight
// and 6 activation fragments for 10 MFMAs.
#include <string.h>

#include <thread>
#include <type_traits>

#include "conv_mfma_common.h"

#define FOLD_TH 8
#define FOLD_PW 36

struct fold_args {
    const __bf16* in;        // t: [N][H][W][CIN]
    const uint4* wp;         // main kernel: middle-class weights [chunk][tap][ks][lane]; ring kernel: all classes
    const float* bias;       // [class][chunk][32]
    float* out;              // [N][s*H][s*W][3]
    const uint32_t* n_valid;
    int N, H, W;
    int s, n_chunks, rows, ipc;   // scale, chunks, valid rows per chunk, output rows i per chunk
    int rev;
    const uint32_t* tile_list;   // the tiles to compute (needed-region mode), or null: all tiles
    const uint32_t* n_list;
};

// Stores the 16 accumulator values of one lane: rows 8q + 4hi + e of chunk `chunk` for
// low-resolution pixel (y, x) of image n.  Row rho of a chunk is (il, j, co) = (rho / 3s, rho / 3 % s,
// rho % 3) with output row i = chunk * ipc + il.
__device__ __forceinline__ void fold_store(const fold_args& a, const f32x16& acc, int n, int y, int x, int chunk, int hi)
{
    const int s = a.s, OW = a.W * s;
    float* base = a.out + (((size_t)n * a.H * s + (size_t)y * s) * OW + (size_t)x * s) * 3;
    if (s == 4) {                      // 12 values per output row i: three aligned groups of four
#pragma unroll
        for (int q = 0; q < 3; ++q) {
            const int rho = 8 * q + 4 * hi, il = rho / 12, off = rho - 12 * il;
            *(float4*)(base + (size_t)(chunk * 2 + il) * OW * 3 + off) = make_float4(acc[4 * q], acc[4 * q + 1], acc[4 * q + 2], acc[4 * q + 3]);
        }
        return;
    }
#pragma unroll
    for (int q = 0; q < 4; ++q)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int rho = 8 * q + 4 * hi + e;
            if (rho >= a.rows) continue;
            const int il = rho / (3 * s), rem = rho - il * 3 * s;
            base[(size_t)(chunk * a.ipc + il) * OW * 3 + rem] = acc[4 * q + e];
        }
}

template <int N, int I = 0, typename F>
__device__ __forceinline__ void fold_each_step(F& f)
{
    if constexpr (I < N) { f(std::integral_constant<int, I>{}); fold_each_step<N, I + 1>(f); }
}

template <int CIN, bool LIST>
__global__ __launch_bounds__(256) void k_conv_fold(fold_args a)
{
    // LIST: the tiles come from a.tile_list.  An entry is requested two tiles ahead with a vector
    // load (a scalar load would share its counter with the LDS fragment reads) and read a tile later.
    constexpr int KS = CIN / 16, NCH = CIN / 8, PIXB = CIN * 2, TH = FOLD_TH, PH = TH + 4, PW = FOLD_PW, RW = 2, NR = RW + 4;
    constexpr int WBYTES = 25 * KS * 1024, NPIECE = PH * PW * NCH, NPRE = (NPIECE + 255) / 256, NSTEP = 5 * KS;
    constexpr int SWZ_SH = (NCH == 8) ? 0 : 1;
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];
    uint8_t* lds_w = lds;
    uint8_t* lds_p = lds + WBYTES;
    const int tid = threadIdx.x, lane = tid & 63, lx = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);

    const int n_img = a.n_valid ? min((int)*a.n_valid, a.N) : a.N;
    const int tiles_x = (a.W + 31) / 32, tiles_y = (a.H + TH - 1) / TH, tiles_img = tiles_x * tiles_y;
    const int n_tiles = LIST ? (int)*a.n_list : n_img * tiles_img;
    // tile lanes and chunks: as in the 3 x 3 kernel, the chunks of a layer are dealt to the workgroups
    // of one XCD that share a tile lane (the input then comes from HBM once), XCD-contiguous tile runs
    const bool deal = a.n_chunks > 1 && gridDim.x % (8 * a.n_chunks) == 0;
    const int G = deal ? gridDim.x / a.n_chunks : gridDim.x;
    const int xcd = blockIdx.x % 8, local = blockIdx.x / 8;
    const int wg = deal ? xcd * (G / 8) + local / a.n_chunks : ((G % 8 == 0) ? xcd * (G / 8) + local : (int)blockIdx.x);
    const int chunk_begin = deal ? local % a.n_chunks : 0, chunk_end = deal ? chunk_begin + 1 : a.n_chunks;
    const uint32_t in_img_bytes = (uint32_t)a.H * a.W * PIXB;

    // patch pieces of this thread: piece j is 16-byte group p_c of patch pixel (p_row, p_col)
    uint4 pre[NPRE];
    auto piece_pos = [&](int j, int& row, int& col, int& c) __attribute__((always_inline)) {
        const int idx = j * 256 + tid, px = idx / NCH;
        c = idx - px * NCH; row = px / PW; col = px - row * PW;
        return idx < NPIECE;
    };
    auto load_piece = [&](int j, __amdgpu_buffer_rsrc_t rin, int y0, int x0) __attribute__((always_inline)) {
        int row, col, c;
        const bool in_patch = piece_pos(j, row, col, c);
        const int gy = y0 - 2 + row, gx = x0 - 2 + col;
        const bool ok = in_patch && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
        const i32x4 v = __builtin_amdgcn_raw_buffer_load_b128(rin, ok ? (uint32_t)((gy * a.W + gx) * PIXB + c * 16) : OOB_OFF, 0, 0);
        pre[j] = make_uint4(v[0], v[1], v[2], v[3]);
    };
    auto store_patch = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int j = 0; j < NPRE; ++j) {
            int row, col, c;
            if (piece_pos(j, row, col, c))
                *(uint4*)(lds_p + (row * PW + col) * PIXB + ((c ^ ((col >> SWZ_SH) & (NCH - 1))) << 4)) = pre[j];
        }
    };
    auto decode = [&](int tile, int& n, int& y0, int& x0) __attribute__((always_inline)) {
        n = tile / tiles_img;
        const int tr = tile - n * tiles_img, ty = tr / tiles_x, tx = tr - ty * tiles_x;
        y0 = ty * TH; x0 = tx * 32;
    };
    __amdgpu_buffer_rsrc_t rlist = __builtin_amdgcn_make_buffer_rsrc((void*)a.tile_list, 0, LIST ? (uint32_t)n_tiles * 4u : 0u, RSRC_FLAGS);
    auto list_load = [&](int idx) __attribute__((always_inline)) {       // entry of walk position idx (0 past the end)
        const int pos = a.rev ? n_tiles - 1 - idx : idx;
        return __builtin_amdgcn_raw_buffer_load_b32(rlist, idx < n_tiles ? (uint32_t)pos * 4u : OOB_OFF, 0, 0);
    };
    auto decode_cell = [&](int cell, int& n, int& y0, int& x0) __attribute__((always_inline)) {    // RH_CELL_ENTRY
        n = (int)((uint32_t)cell >> 16); y0 = (int)(((uint32_t)cell >> 7) & 511u) * TH; x0 = (int)((uint32_t)cell & 127u) * 32;
    };
    auto tile_origin = [&](int tile, int& n, int& y0, int& x0) __attribute__((always_inline)) {
        if constexpr (LIST) { decode_cell(__builtin_amdgcn_readfirstlane(list_load(tile)), n, y0, x0); return; }
        if (a.rev && tile < n_tiles) tile = n_tiles - 1 - tile;          // walk back over what the previous layer wrote last
        decode(tile, n, y0, x0);
    };
    auto in_rsrc = [&](int tile, int n) __attribute__((always_inline)) {
        return __builtin_amdgcn_make_buffer_rsrc((void*)(a.in + (size_t)n * a.H * a.W * CIN), 0,
                                                 tile < n_tiles ? in_img_bytes : 0u, RSRC_FLAGS);
    };

    for (int chunk = chunk_begin; chunk < chunk_end; ++chunk) {
        __syncthreads();                                   // previous chunk's LDS reads are done
        {
            const uint4* src = a.wp + (size_t)chunk * (WBYTES / 16);
            for (int i = tid; i < WBYTES / 16; i += 256) ((uint4*)lds_w)[i] = src[i];
        }
        f32x16 biasv;                                      // lane holds rows 8q + 4hi + e in [4q + e]
#pragma unroll
        for (int e = 0; e < 16; ++e) biasv[e] = a.bias[chunk * 32 + (e >> 2) * 8 + hi * 4 + (e & 3)];
        int tile = wg;
        int cn = 0, cy0 = 0, cx0 = 0, e_next = 0;         // LIST: origin of the current tile, entry of the next one
        {
            int n, y0, x0; tile_origin(tile, n, y0, x0);
            cn = n; cy0 = y0; cx0 = x0;
            if constexpr (LIST) e_next = list_load(tile + G);
            __amdgpu_buffer_rsrc_t rin = in_rsrc(tile, tile < n_tiles ? n : 0);
#pragma unroll
            for (int j = 0; j < NPRE; ++j) load_piece(j, rin, y0, x0);
        }
        for (; tile < n_tiles; tile += G) {                // trip count uniform over the workgroup
            int n, y0, x0;
            if constexpr (LIST) { n = cn; y0 = cy0; x0 = cx0; } else tile_origin(tile, n, y0, x0);
            int e_after = 0;
            if constexpr (LIST) e_after = list_load(tile + 2 * G);
            lds_barrier();                                 // LDS reads of the previous tile are done
            store_patch();
            lds_barrier();
            const int nt = tile + G;
            int nn, ny0, nx0;
            if constexpr (LIST) { decode_cell(__builtin_amdgcn_readfirstlane(e_next), nn, ny0, nx0); cn = nn; cy0 = ny0; cx0 = nx0; e_next = e_after; }
            else tile_origin(nt, nn, ny0, nx0);
            __amdgpu_buffer_rsrc_t rin = in_rsrc(nt, nt < n_tiles ? nn : 0);

            f32x16 acc[RW];
#pragma unroll
            for (int r = 0; r < RW; ++r) acc[r] = biasv;
            const uint8_t* wlane = lds_w + (lane << 4);
            const uint8_t* prow = lds_p + (wave * RW) * (PW * PIXB);
            bf16x8 A0[5], A1[5], B0[NR], B1[NR];
            auto load_frags = [&](int st, bf16x8 (&A)[5], bf16x8 (&B)[NR]) __attribute__((always_inline)) {
                const int kx = st / KS, ks = st - kx * KS, px = lx + kx;
                const uint8_t* b0 = prow + px * PIXB + (((2 * ks + hi) ^ ((px >> SWZ_SH) & (NCH - 1))) << 4);
#pragma unroll
                for (int ky = 0; ky < 5; ++ky) A[ky] = *(const bf16x8*)(wlane + ((((ky * 5 + kx) * KS) + ks) << 10));
#pragma unroll
                for (int py = 0; py < NR; ++py) B[py] = *(const bf16x8*)(b0 + py * (PW * PIXB));
            };
            load_frags(0, A0, B0);
            auto step = [&](auto st_c) __attribute__((always_inline)) {
                constexpr int st = decltype(st_c)::value;
                bf16x8 (&Ac)[5] = (st & 1) ? A1 : A0;
                bf16x8 (&Bc)[NR] = (st & 1) ? B1 : B0;
                bf16x8 (&An)[5] = (st & 1) ? A0 : A1;
                bf16x8 (&Bn)[NR] = (st & 1) ? B0 : B1;
                if constexpr (st + 1 < NSTEP) load_frags(st + 1, An, Bn);
                if constexpr (st < NPRE) load_piece(st, rin, ny0, nx0);        // next tile's patch, one piece per step
                static_assert(NPRE <= NSTEP, "one patch piece per step must cover the patch");
                __builtin_amdgcn_sched_barrier(0);
                // (input row py, tap row ky) pairs with 0 <= py - ky < RW
#pragma unroll
                for (int py = 0; py < NR; ++py)
#pragma unroll
                    for (int ky = 0; ky < 5; ++ky)
                        if (py - ky >= 0 && py - ky < RW)
                            acc[py - ky] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(Ac[ky], Bc[py], acc[py - ky], 0, 0, 0);
                __builtin_amdgcn_sched_barrier(0);
            };
            fold_each_step<NSTEP>(step);
            const int x = x0 + lx;
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                const int y = y0 + wave * RW + r;
                if (y < a.H && x < a.W) fold_store(a, acc[r], n, y, x, chunk, hi);
            }
        }
    }
}

// The outermost ring of every image again, with the weights of its position class.  One wave per
// (class, 32 ring pixels, chunk): operands straight from global memory (the ring is 3 % of the pixels).
// Classes are numbered 3 * (0 top / 1 middle / 2 bottom) + (0 left / 1 middle / 2 right).
template <int CIN>
__global__ __launch_bounds__(64) void k_fold_ring(fold_args a)
{
    constexpr int KS = CIN / 16;
    const int lane = threadIdx.x, lx = lane & 31, hi = lane >> 5;
    const int chunk = blockIdx.z;
    const int cls_tab[8] = {1, 7, 3, 5, 0, 2, 6, 8};       // top, bottom, left, right edges, then the corners
    const int kind = blockIdx.y, cls = cls_tab[kind];
    const int n_img = a.n_valid ? min((int)*a.n_valid, a.N) : a.N;
    const int per = kind < 2 ? a.W - 2 : (kind < 4 ? a.H - 2 : 1);      // ring pixels of this class per image
    const long total = (long)n_img * per;
    if ((long)blockIdx.x * 32 >= total) return;
    const long q = (long)blockIdx.x * 32 + lx;
    const bool valid = q < total;
    const int n = valid ? (int)(q / per) : 0, k = valid ? (int)(q - (long)n * per) : 0;
    int y, x;
    switch (kind) {
        case 0: y = 0; x = 1 + k; break;
        case 1: y = a.H - 1; x = 1 + k; break;
        case 2: y = 1 + k; x = 0; break;
        case 3: y = 1 + k; x = a.W - 1; break;
        case 4: y = 0; x = 0; break;
        case 5: y = 0; x = a.W - 1; break;
        case 6: y = a.H - 1; x = 0; break;
        default: y = a.H - 1; x = a.W - 1; break;
    }
    const uint4* wp = a.wp + (size_t)(cls * a.n_chunks + chunk) * (25 * KS * 64);
    const float* bias = a.bias + (cls * a.n_chunks + chunk) * 32;
    f32x16 acc;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[e] = bias[(e >> 2) * 8 + hi * 4 + (e & 3)];
    const __bf16* img = a.in + (size_t)n * a.H * a.W * CIN;
    // one tap row (5 taps x KS k-steps) of operands is requested while the previous one is multiplied:
    // a wave that waited for every tap's loads in turn spent 100 load latencies per pixel group
    uint4 A[2][5][KS], B[2][5][KS];
    auto load_row = [&](int ky, uint4 (&Ar)[5][KS], uint4 (&Br)[5][KS]) __attribute__((always_inline)) {
        const int yy = y + ky - 2;
        const bool row_ok = valid && yy >= 0 && yy < a.H;
#pragma unroll
        for (int kx = 0; kx < 5; ++kx) {
            const int xx = x + kx - 2;
            const bool ok = row_ok && xx >= 0 && xx < a.W;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                Ar[kx][ks] = wp[((ky * 5 + kx) * KS + ks) * 64 + lane];
                Br[kx][ks] = ok ? *(const uint4*)(img + ((size_t)yy * a.W + xx) * CIN + ks * 16 + hi * 8) : make_uint4(0, 0, 0, 0);
            }
        }
    };
    load_row(0, A[0], B[0]);
#pragma unroll
    for (int ky = 0; ky < 5; ++ky) {
        if (ky + 1 < 5) load_row(ky + 1, A[(ky + 1) & 1], B[(ky + 1) & 1]);
#pragma unroll
        for (int kx = 0; kx < 5; ++kx)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(*(const bf16x8*)&A[ky & 1][kx][ks], *(const bf16x8*)&B[ky & 1][kx][ks], acc, 0, 0, 0);
    }
    if (valid) fold_store(a, acc, n, y, x, chunk, hi);
}

// ------------------------------------------------------------------------------------------
// host side: composition of the layers' weights

namespace {

struct fold_stage { const float* w; const float* b; int cin, cout, r; };   // conv3x3 cin -> cout, then pixel shuffle by r

// Gradient of output (Yf, Xf, co) of the last stage's conv with respect to the first stage's input,
// on a small image whose first-stage grid is g0 x g0 (zero padding at every stage's own border).
// grid[k] = side of stage k's input grid.
void fold_gradient(const std::vector<fold_stage>& st, const std::vector<int>& grid, int Yf, int Xf, int co,
                   std::vector<double>& g_in0)
{
    const int K = (int)st.size();
    std::vector<double> gc((size_t)grid[K - 1] * grid[K - 1] * st[K - 1].cout, 0.0);
    gc[((size_t)Yf * grid[K - 1] + Xf) * st[K - 1].cout + co] = 1.0;
    int cy0 = Yf, cy1 = Yf, cx0 = Xf, cx1 = Xf;            // bounding box of the non-zeros of gc
    for (int k = K - 1; k >= 0; --k) {
        const fold_stage& S = st[k];
        const int g = grid[k];
        std::vector<double> gi((size_t)g * g * S.cin, 0.0);
        for (int y = cy0; y <= cy1; ++y) for (int x = cx0; x <= cx1; ++x) for (int c = 0; c < S.cout; ++c) {
            const double v = gc[((size_t)y * g + x) * S.cout + c];
            if (v == 0.0) continue;
            for (int ky = 0; ky < 3; ++ky) {
                const int iy = y + ky - 1; if (iy < 0 || iy >= g) continue;      // zero padding: no input there
                for (int kx = 0; kx < 3; ++kx) {
                    const int ix = x + kx - 1; if (ix < 0 || ix >= g) continue;
                    const float* w = S.w + (((size_t)c * 3 + ky) * 3 + kx) * S.cin;
                    double* d = &gi[((size_t)iy * g + ix) * S.cin];
                    for (int ci = 0; ci < S.cin; ++ci) d[ci] += v * (double)w[ci];
                }
            }
        }
        const int iy0 = std::max(cy0 - 1, 0), iy1 = std::min(cy1 + 1, g - 1), ix0 = std::max(cx0 - 1, 0), ix1 = std::min(cx1 + 1, g - 1);
        if (k == 0) { g_in0.swap(gi); return; }
        // back through the previous stage's pixel shuffle: ps[y*r+i][x*r+j][c] = conv[y][x][c*r*r + i*r + j]
        const fold_stage& P = st[k - 1];
        const int r = P.r, gp = grid[k - 1];
        gc.assign((size_t)gp * gp * P.cout, 0.0);
        for (int y = iy0; y <= iy1; ++y) for (int x = ix0; x <= ix1; ++x) for (int c = 0; c < S.cin; ++c) {
            const double v = gi[((size_t)y * g + x) * S.cin + c];
            if (v != 0.0) gc[((size_t)(y / r) * gp + x / r) * P.cout + c * r * r + (y % r) * r + (x % r)] = v;
        }
        cy0 = iy0 / r; cy1 = iy1 / r; cx0 = ix0 / r; cx1 = ix1 / r;
    }
}

// The stages' response to an all-zero input on the small image (the composite bias at every position).
void fold_bias(const std::vector<fold_stage>& st, const std::vector<int>& grid, std::vector<double>& out /*[g][g][cout_last]*/)
{
    std::vector<double> x((size_t)grid[0] * grid[0] * st[0].cin, 0.0);
    for (size_t k = 0; k < st.size(); ++k) {
        const fold_stage& S = st[k];
        const int g = grid[k];
        std::vector<double> yv((size_t)g * g * S.cout);
        for (int y = 0; y < g; ++y) for (int xx = 0; xx < g; ++xx) for (int c = 0; c < S.cout; ++c) {
            double acc = (double)S.b[c];
            for (int ky = 0; ky < 3; ++ky) {
                const int iy = y + ky - 1; if (iy < 0 || iy >= g) continue;
                for (int kx = 0; kx < 3; ++kx) {
                    const int ix = xx + kx - 1; if (ix < 0 || ix >= g) continue;
                    const float* w = S.w + (((size_t)c * 3 + ky) * 3 + kx) * S.cin;
                    const double* in = &x[((size_t)iy * g + ix) * S.cin];
                    for (int ci = 0; ci < S.cin; ++ci) acc += (double)w[ci] * in[ci];
                }
            }
            yv[((size_t)y * g + xx) * S.cout + c] = acc;
        }
        if (S.r == 1) { x.swap(yv); continue; }
        const int r = S.r, co = S.cout / (r * r);
        x.assign((size_t)g * r * g * r * co, 0.0);
        for (int y = 0; y < g; ++y) for (int xx = 0; xx < g; ++xx) for (int c = 0; c < co; ++c)
            for (int i = 0; i < r; ++i) for (int j = 0; j < r; ++j)
                x[((size_t)(y * r + i) * (g * r) + (xx * r + j)) * co + c] = yv[((size_t)y * g + xx) * S.cout + c * r * r + i * r + j];
    }
    out.swap(x);
}

uint16_t fold_bf16(double v)
{
    const float f = (float)v;
    uint32_t u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

}  // namespace

// Builds ctx->fold_w / fold_b for an EDSR-shaped net; a no-op for the other topologies.
// Layout: fold_w [class 9][chunk][tap 25][ks][lane 64][8] bf16 with row = lane % 32 of the chunk and
// ci = 16 ks + 8 (lane / 32) + e; fold_b [class][chunk][32] fp32.
rh_status rh_fold_weights(rh_ctx* ctx, const float* blob)
{
    const rh_net_desc& d = ctx->cfg.net;
    ctx->fold_chunks = 0;
    if (d.topology != RH_NET_EDSR || ctx->cfg.precision != RH_BF16) return RH_OK;
    const int C = d.channels, s = d.scale;
    if (C != 32 && C != 64) return RH_OK;
    const size_t nl = ctx->layers.size();
    std::vector<fold_stage> st;
    const int n_up = s == 4 ? 2 : 1;
    for (int u = 0; u < n_up; ++u) {
        const rh_layer& L = ctx->layers[nl - 1 - n_up + u];
        st.push_back({blob + L.w_off, blob + L.b_off, L.cin, L.cout, s == 4 ? 2 : s});
    }
    const rh_layer& T = ctx->layers[nl - 1];
    st.push_back({blob + T.w_off, blob + T.b_off, T.cin, T.cout, 1});
    std::vector<int> grid(st.size());
    grid[0] = 5;
    for (size_t k = 1; k < st.size(); ++k) grid[k] = grid[k - 1] * st[k - 1].r;
    const int gl = grid.back();                            // = 5 s
    const int R = 3 * s * s, n_chunks = s == 4 ? 2 : 1, ipc = s == 4 ? 2 : s, rows = 3 * s * ipc, KS = C / 16;
    std::vector<double> bias_all;
    fold_bias(st, grid, bias_all);
    // Wc[class][i][j][co][tap][ci]; the class's pixel sits at row / column 0, 2 or 4 of the 5 x 5 image
    std::vector<double> Wc((size_t)9 * R * 25 * C, 0.0);
    auto work = [&](int job0, int job1) {
        std::vector<double> g;
        for (int job = job0; job < job1; ++job) {
            const int cls = job / R, o = job - cls * R, py = 2 * (cls / 3), px = 2 * (cls % 3);
            const int i = o / (3 * s), j = (o / 3) % s, co = o % 3;
            fold_gradient(st, grid, py * s + i, px * s + j, co, g);
            double* dst = &Wc[((size_t)cls * R + o) * 25 * C];
            for (int dy = -2; dy <= 2; ++dy) for (int dx = -2; dx <= 2; ++dx) {
                const int yy = py + dy, xx = px + dx;
                if (yy < 0 || yy >= 5 || xx < 0 || xx >= 5) continue;           // outside the image: t is zero there
                memcpy(dst + ((dy + 2) * 5 + (dx + 2)) * C, &g[((size_t)yy * 5 + xx) * C], sizeof(double) * C);
            }
        }
    };
    {
        const int jobs = 9 * R, nt = 8;
        std::vector<std::thread> th;
        for (int t = 0; t < nt; ++t) th.emplace_back(work, jobs * t / nt, jobs * (t + 1) / nt);
        for (auto& t : th) t.join();
    }
    std::vector<uint16_t> wp((size_t)9 * n_chunks * 25 * KS * 64 * 8);
    std::vector<float> bp((size_t)9 * n_chunks * 32, 0.0f);
    size_t wi = 0;
    for (int cls = 0; cls < 9; ++cls)
        for (int m = 0; m < n_chunks; ++m) {
            const int py = 2 * (cls / 3), px = 2 * (cls % 3);
            for (int tap = 0; tap < 25; ++tap)
                for (int ks = 0; ks < KS; ++ks)
                    for (int lane = 0; lane < 64; ++lane)
                        for (int e = 0; e < 8; ++e) {
                            const int rho = lane & 31, ci = ks * 16 + 8 * (lane >> 5) + e;
                            double v = 0.0;
                            if (rho < rows) {
                                const int il = rho / (3 * s), rem = rho - il * 3 * s, o = (m * ipc + il) * 3 * s + rem;
                                v = Wc[(((size_t)cls * R + o) * 25 + tap) * C + ci];
                            }
                            wp[wi++] = fold_bf16(v);
                        }
            for (int rho = 0; rho < rows; ++rho) {
                const int il = rho / (3 * s), rem = rho - il * 3 * s, i = m * ipc + il, j = rem / 3, co = rem % 3;
                bp[((size_t)cls * n_chunks + m) * 32 + rho] = (float)bias_all[((size_t)(py * s + i) * gl + (px * s + j)) * 3 + co];
            }
        }
    RH_HIP(ctx, hipMalloc(&ctx->fold_w, wp.size() * 2));
    RH_HIP(ctx, hipMalloc((void**)&ctx->fold_b, bp.size() * 4));
    RH_HIP(ctx, hipMemcpy(ctx->fold_w, wp.data(), wp.size() * 2, hipMemcpyHostToDevice));
    RH_HIP(ctx, hipMemcpy(ctx->fold_b, bp.data(), bp.size() * 4, hipMemcpyHostToDevice));
    ctx->fold_chunks = n_chunks; ctx->fold_rows = rows; ctx->fold_ipc = ipc;
    return RH_OK;
}

template <int CIN>
static hipError_t launch_fold(rh_ctx* ctx, const fold_args& a)
{
    constexpr int lds = 25 * (CIN / 16) * 1024 + (FOLD_TH + 4) * FOLD_PW * CIN * 2;
    static bool attr_done[RH_MAX_DEVICES] = {};
    if (!attr_done[ctx->device]) {
        hipError_t e = hipFuncSetAttribute((const void*)k_conv_fold<CIN, false>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e == hipSuccess) e = hipFuncSetAttribute((const void*)k_conv_fold<CIN, true>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_done[ctx->device] = true;
    }
    fold_args m = a;                                       // main kernel: the middle class (number 4)
    m.wp = a.wp + (size_t)4 * a.n_chunks * (25 * (CIN / 16) * 64);
    m.bias = a.bias + 4 * a.n_chunks * 32;
    if (a.tile_list) hipLaunchKernelGGL((k_conv_fold<CIN, true>), dim3(ctx->n_cu), dim3(256), lds, ctx->stream, m);
    else hipLaunchKernelGGL((k_conv_fold<CIN, false>), dim3(ctx->n_cu), dim3(256), lds, ctx->stream, m);
    // Needed-region mode: a pasted macroblock lies at least `halo` pixels inside its box, hence inside
    // the bin, so with a halo no pasted pixel is on the outermost ring and the ring pass has nothing to add.
    if (a.tile_list && ctx->cfg.halo >= 1) return hipGetLastError();
    const long longest = (long)a.N * (a.W > a.H ? a.W : a.H);
    const long groups = (longest + 31) / 32;
    if (groups > 0x7FFFFFFFL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_fold_ring<CIN>, dim3((unsigned)groups, 8, a.n_chunks), dim3(64), 0, ctx->stream, a);
    return hipGetLastError();
}

// t: the body's output [N][H][W][C] bf16 -> raw network output fp32 [N][sH][sW][3]; two launches.
rh_status rh_launch_fold(rh_ctx* ctx, const __bf16* t, float* out, int N, int H, int W, const uint32_t* n_valid, int rev,
                         const uint32_t* tile_list, const uint32_t* n_list)
{
    fold_args a;
    a.tile_list = tile_list; a.n_list = n_list;
    a.in = t; a.wp = (const uint4*)ctx->fold_w; a.bias = ctx->fold_b; a.out = out; a.n_valid = n_valid;
    a.N = N; a.H = H; a.W = W; a.s = ctx->cfg.net.scale; a.n_chunks = ctx->fold_chunks; a.rows = ctx->fold_rows;
    a.ipc = ctx->fold_ipc; a.rev = rev;
    const int C = ctx->cfg.net.channels;
    RH_HIP(ctx, C == 64 ? launch_fold<64>(ctx, a) : launch_fold<32>(ctx, a));
    return RH_OK;
}

// First conv of the network (Sec. 3.3.3: the enhancement model applied to the packed bins):
// 3 input channels read from the u8 image, C output channels, bf16 NHWC result.
//
// K = 27 is short, so the cost of a matrix-core formulation is building the B operand.  Here the
// u8 patch of an 8 x 32 tile is converted once (x/255 rounded to bf16, through a 256-entry table)
// and expanded in LDS into one 16-value record per (patch row, pixel): the 9 values
// [kx][c] of that row under the pixel's 3 x 3 window, then 7 zeros.  With K ordered as
// ky*16 + kx*3 + c a B fragment is one aligned 16-byte LDS read per ky (3 k-steps of 16, 9 of
// each used), and the accumulators start from the bias.  The result leaves through a wave-private
// LDS slice so that stores move whole 2C-byte pixels.
#include "conv_mfma_common.h"

#define HEAD_TH 8
#define HEAD_RUN 32

template <int C>
__global__ __launch_bounds__(256) void k_head_mfma(const uint8_t* __restrict__ in, const uint4* __restrict__ wp /*[3][MT][64]*/,
                                                   const float* __restrict__ bias, __bf16* __restrict__ out, int N, int H,
                                                   int W, int relu, const uint32_t* __restrict__ n_valid)
{
    constexpr int MT = C / 32, PH = HEAD_TH + 2, PWB = 34 * 3, OPIXB = C * 2, NCHO = OPIXB / 16;
    constexpr int PPJ = 64 / NCHO, NOUT = 2 * 32 / PPJ;                  // pixels per store instruction, stores per wave
    __shared__ __attribute__((aligned(16))) uint8_t s_raw[PH * PWB + 4];  // u8 patch, rows of 34 pixels
    __shared__ __attribute__((aligned(16))) uint16_t s_lut[256];          // bf16(x / 255)
    __shared__ __attribute__((aligned(16))) uint16_t s_rec[PH * 32 * 16]; // expanded records
    __shared__ __attribute__((aligned(16))) uint8_t s_stg[4 * 2 * 32 * OPIXB];
    const int tid = threadIdx.x, lane = tid & 63, lx = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // uniform over the wave: keeps row indices scalar

    const int n_img = n_valid ? min((int)*n_valid, N) : N;
    const int tiles_x = (W + 31) / 32, tiles_y = (H + HEAD_TH - 1) / HEAD_TH, tiles_img = tiles_x * tiles_y;
    const int n_tiles = n_img * tiles_img;
    // XCD-aware order: each XCD takes runs of HEAD_RUN consecutive tiles, all XCDs stay close together
    const int b = blockIdx.x, grp = b / (8 * HEAD_RUN), in_grp = b - grp * (8 * HEAD_RUN);
    const int tile = grp * (8 * HEAD_RUN) + (in_grp % 8) * HEAD_RUN + in_grp / 8;
    if (tile >= n_tiles) return;                                          // uniform over the workgroup
    const int n = tile / tiles_img, tr = tile - n * tiles_img, ty = tr / tiles_x, tx = tr - ty * tiles_x;
    const int y0 = ty * HEAD_TH, x0 = tx * 32;
    const uint8_t* img = in + (size_t)n * H * W * 3;

    {   // table and raw patch (zero outside the image = zero padding: bf16(0/255) = 0)
        const float f = __fdiv_rn((float)tid, 255.0f);
        s_lut[tid] = (uint16_t)(pack_bf16x2(f, 0.0f) & 0xFFFFu);
        for (int i = tid; i < PH * PWB; i += 256) {
            const int row = i / PWB, cb = i - row * PWB, col = cb / 3, ch = cb - col * 3;
            const int gy = y0 - 1 + row, gx = x0 - 1 + col;
            s_raw[i] = (gy >= 0 && gy < H && gx >= 0 && gx < W) ? img[((size_t)gy * W + gx) * 3 + ch] : (uint8_t)0;
        }
    }
    __syncthreads();
    // expand: record (row, px) = the 9 converted bytes starting at patch column px, then zeros
    for (int r = tid; r < PH * 32; r += 256) {
        const int row = r >> 5, px = r & 31;
        const uint8_t* src = s_raw + row * PWB + px * 3;
        uint32_t v[8];
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = (uint32_t)s_lut[src[2 * j]] | ((uint32_t)s_lut[src[2 * j + 1]] << 16);
        v[4] = (uint32_t)s_lut[src[8]];
        v[5] = v[6] = v[7] = 0u;
        uint4* dst = (uint4*)(s_rec + r * 16);
        dst[0] = make_uint4(v[0], v[1], v[2], v[3]);
        dst[1] = make_uint4(v[4], v[5], v[6], v[7]);
    }
    bf16x8 A[3][MT];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky)
#pragma unroll
        for (int m = 0; m < MT; ++m) { const uint4 v = wp[(ky * MT + m) * 64 + lane]; A[ky][m] = *(const bf16x8*)&v; }
    float bv[MT][16];
#pragma unroll
    for (int m = 0; m < MT; ++m)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e) bv[m][4 * q + e] = bias[m * 32 + 8 * q + 4 * hi + e];
    __syncthreads();

    uint8_t* stg = s_stg + wave * (2 * 32 * OPIXB);
    const int okey = lx & (NCHO - 1);
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        const int row = wave * 2 + r;                                     // output row inside the tile
        f32x16 acc[MT];
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[m][e] = bv[m][e];
#pragma unroll
        for (int ky = 0; ky < 3; ++ky) {
            const bf16x8 B = *(const bf16x8*)(s_rec + ((row + ky) * 32 + lx) * 16 + hi * 8);
#pragma unroll
            for (int m = 0; m < MT; ++m) acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[ky][m], B, acc[m], 0, 0, 0);
        }
        // lane holds channels m*32 + 8q + 4hi + {0..3} of pixel lx in acc[m][4q..4q+3]
#pragma unroll
        for (int m = 0; m < MT; ++m)
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float v0 = acc[m][4 * q], v1 = acc[m][4 * q + 1], v2 = acc[m][4 * q + 2], v3 = acc[m][4 * q + 3];
                uint2 pk;
                pk.x = pack_bf16x2(v0, v1); pk.y = pack_bf16x2(v2, v3);
                if (relu) { pk.x = relu_bf16x2(pk.x); pk.y = relu_bf16x2(pk.y); }
                *(uint2*)(stg + (r * 32 + lx) * OPIXB + (((m * 4 + q) ^ okey) << 4) + hi * 8) = pk;
            }
    }
    // the slice is private to the wave: no barrier, only the wave's own LDS writes must have landed
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    const int lcol = lane / NCHO, lc = lane % NCHO;
#pragma unroll
    for (int j = 0; j < NOUT; ++j) {
        const int p = j * PPJ + lcol, r = p >> 5, px = p & 31;            // 64 pixels of the wave's two rows
        const int y = y0 + wave * 2 + r, x = x0 + px;
        const uint4 o = *(const uint4*)(stg + (r * 32 + px) * OPIXB + ((lc ^ (px & (NCHO - 1))) << 4));
        if (y < H && x < W) *(uint4*)((uint8_t*)out + (((size_t)n * H + y) * W + x) * OPIXB + lc * 16) = o;
    }
}

template <int C>
static hipError_t launch_head(hipStream_t stream, const uint8_t* in, const uint4* wp, const float* bias, __bf16* out, int N,
                              int H, int W, int relu, const uint32_t* n_valid)
{
    const long long tiles = (long long)N * ((H + HEAD_TH - 1) / HEAD_TH) * ((W + 31) / 32);
    const long long grid = (tiles + 8 * HEAD_RUN - 1) / (8 * HEAD_RUN) * (8 * HEAD_RUN);
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(k_head_mfma<C>, dim3((unsigned)grid), dim3(256), 0, stream, in, wp, bias, out, N, H, W, relu, n_valid);
    return hipGetLastError();
}

// wp: [ky 3][m C/32][64 lanes][8] bf16 with cout = m*32 + lane%32 and k = 8*(lane/32) + e = kx*3 + c (k >= 9: zero)
hipError_t rh_launch_head_mfma(hipStream_t stream, int C, const uint8_t* in, const uint4* wp, const float* bias, __bf16* out,
                               int N, int H, int W, int relu, const uint32_t* n_valid)
{
    if (C == 64) return launch_head<64>(stream, in, wp, bias, out, N, H, W, relu, n_valid);
    if (C == 32) return launch_head<32>(stream, in, wp, bias, out, N, H, W, relu, n_valid);
    return hipErrorInvalidValue;
}

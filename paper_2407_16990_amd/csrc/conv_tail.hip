// Last conv of the EDSR-shaped nets (Sec. 3.3: the enhancement model applied to the packed
// bins): CIN -> 3 channels at the output resolution, fp32 result.
//
// With 3 output channels a conv3x3 as one implicit GEMM over K = 9*CIN wastes most of an MFMA
// tile's rows, and every input pixel vector is read nine times.  Here the conv is split into
//   (1) a 1x1 contraction   P[q][tap*3 + co] = sum_ci  w[co][tap][ci] * x[q][ci]
//       over the (TH+2) x 34 pixel patch of a TH x 32 output tile: M = 27 (padded to 32) rows,
//       N = 32 pixels, K = CIN, on the matrix cores (each pixel vector is fetched once and read
//       from LDS once);
//   (2) a 9-term shifted sum  out[y][x][co] = bias[co] + sum_tap P[(y+ky, x+kx)][tap*3 + co]
//       on the vector ALU, from P kept in LDS as fp32, taps added in ascending order.
// Pixels outside the image contribute P = 0, which is the per-layer zero padding.
// The kernel is a stream over the input tensor: 2*CIN bytes read and 12 bytes written per pixel.
#include "conv_mfma_common.h"

#define TAIL_PW 34
#define TAIL_RUN 32
#define TAIL_PITCH 144          // bytes per patch pixel in LDS: 32 floats + 4 pad (two-way bank conflicts at most)

template <int CIN, int TH>
__global__ __launch_bounds__(256) void k_conv_tail3(conv_args a, int tpb /* consecutive tiles per workgroup */)
{
    constexpr int KS = CIN / 16, PIXB = CIN * 2, PH = TH + 2, NQ = PH * TAIL_PW, NT = (NQ + 31) / 32, TPW = (NT + 3) / 4;
    constexpr int NPP = PIXB / 16, NPL = (NQ * NPP + 255) / 256;       // pieces per pixel, pieces per thread
    extern __shared__ __attribute__((aligned(16))) uint8_t lds[];      // NT * 32 rows of TAIL_PITCH bytes
    const int tid = threadIdx.x, lane = tid & 63, lx = lane & 31, hi = lane >> 5;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);          // uniform over the wave: keeps row indices scalar

    const int n_img = a.n_valid ? min((int)*a.n_valid, a.N) : a.N;
    const int tiles_x = (a.W + 31) / 32, tiles_y = (a.H + TH - 1) / TH, tiles_img = tiles_x * tiles_y;
    const int n_tiles = n_img * tiles_img;
    // Workgroups go to the 8 XCDs round-robin.  Within every group of 8*TAIL_RUN workgroups each
    // XCD takes a run of TAIL_RUN consecutive tile sets, so that tiles sharing halo pixels meet in
    // one L2 while all XCDs stay in the same neighbourhood of the tensor (XCDs working megabytes
    // apart at power-of-two offsets collide on the same memory channels).
    const int b = blockIdx.x, grp = b / (8 * TAIL_RUN), in_grp = b - grp * (8 * TAIL_RUN);
    const int tile0 = (grp * (8 * TAIL_RUN) + (in_grp % 8) * TAIL_RUN + in_grp / 8) * tpb;

    bf16x8 A[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) { const uint4 v = a.wp[ks * 64 + lane]; A[ks] = *(const bf16x8*)&v; }
    const float b0 = a.bias[0], b1 = a.bias[1], b2 = a.bias[2];

    for (int tile_i = tile0; tile_i < tile0 + tpb && tile_i < n_tiles; ++tile_i) {   // trip count uniform over the workgroup
    // a.rev: walk the tensor from its end, where the layer before (walking the other way) has just
    // written it and it still sits in the memory-side cache
    const int tile = a.rev ? n_tiles - 1 - tile_i : tile_i;
    const int n = tile / tiles_img, tr = tile - n * tiles_img, ty = tr / tiles_x, tx = tr - ty * tiles_x;
    const int y0 = ty * TH, x0 = tx * 32;

    // (0) the patch goes to LDS in 16-byte pieces, NPP consecutive lanes per pixel vector so that
    //     every load instruction covers whole cache lines; piece c of pixel q sits in slot c ^ (q % NPP)
    const uint32_t img_bytes = (uint32_t)a.H * a.W * PIXB;
    __amdgpu_buffer_rsrc_t rin = __builtin_amdgcn_make_buffer_rsrc((void*)((uint8_t*)a.in + (size_t)n * img_bytes), 0, img_bytes, RSRC_FLAGS);
    i32x4 pre[NPL];
#pragma unroll
    for (int j = 0; j < NPL; ++j) {
        const int pidx = j * 256 + tid, q = pidx / NPP, c = pidx - q * NPP;
        const int row = q / TAIL_PW, col = q - row * TAIL_PW, gy = y0 - 1 + row, gx = x0 - 1 + col;
        const bool ok = q < NQ && gy >= 0 && gy < a.H && gx >= 0 && gx < a.W;
        pre[j] = __builtin_amdgcn_raw_buffer_load_b128(rin, ok ? (uint32_t)((gy * a.W + gx) * PIXB + c * 16) : OOB_OFF, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < NPL; ++j) {
        const int pidx = j * 256 + tid, q = pidx / NPP, c = pidx - q * NPP;
        if (q < NQ) *(i32x4*)(lds + q * PIXB + ((c ^ (q & (NPP - 1))) << 4)) = pre[j];
    }
    __syncthreads();
    // (1) B fragments of this wave's pixel groups: lane (lx, hi) holds channels 16*ks + 8*hi .. +7 of
    //     patch pixel 32*t + lx.  (Pixels NQ.. of the last group are never used.)
    bf16x8 B[TPW][KS];
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int t = wave + 4 * i, q = 32 * t + lx;
        if (t < NT) {
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) B[i][ks] = *(const bf16x8*)(lds + q * PIXB + (((2 * ks + hi) ^ (q & (NPP - 1))) << 4));
        }
    }
    __syncthreads();                                                    // P overwrites the patch
#pragma unroll
    for (int i = 0; i < TPW; ++i) {
        const int t = wave + 4 * i, q = 32 * t + lx;
        if (t < NT) {                                                   // uniform over the wave
            f32x16 acc;
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[e] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(A[ks], B[i][ks], acc, 0, 0, 0);
            // lane holds rows 8g + 4hi + {0..3} of column lx in acc[4g..4g+3]
#pragma unroll
            for (int g = 0; g < 4; ++g)
                *(float4*)(lds + q * TAIL_PITCH + (8 * g + 4 * hi) * 4) = make_float4(acc[4 * g], acc[4 * g + 1], acc[4 * g + 2], acc[4 * g + 3]);
        }
    }
    __syncthreads();

#pragma unroll
    for (int p0 = 0; p0 < TH * 32; p0 += 256) {
        const int p = p0 + tid, oy = p >> 5, ox = p & 31;
        const int y = y0 + oy, x = x0 + ox;
        float o0 = b0, o1 = b1, o2 = b2;
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const float* P = (const float*)(lds + ((oy + ky) * TAIL_PW + ox + kx) * TAIL_PITCH) + (ky * 3 + kx) * 3;
                o0 += P[0]; o1 += P[1]; o2 += P[2];
            }
        if (oy < TH && y < a.H && x < a.W) {
            float* o = (float*)a.out + (((size_t)n * a.H + y) * a.W + x) * 3;
            o[0] = o0; o[1] = o1; o[2] = o2;
        }
    }
    __syncthreads();                                                    // P is free for the next patch
    }
}

template <int CIN, int TH>
static hipError_t launch_tail(hipStream_t stream, int device, const conv_args& a)
{
    constexpr int NQ = (TH + 2) * TAIL_PW, NT = (NQ + 31) / 32, lds = NT * 32 * TAIL_PITCH;
    static bool attr_done[RH_MAX_DEVICES] = {};            // the attribute is per device
    if (!attr_done[device]) {
        hipError_t e = hipFuncSetAttribute((const void*)k_conv_tail3<CIN, TH>, hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
        attr_done[device] = true;
    }
    const long long tiles = (long long)a.N * ((a.H + TH - 1) / TH) * ((a.W + 31) / 32);
    // several consecutive tiles per workgroup once there are enough tiles to fill the chip
    // (measured on 76 x 512 x 512 x 64: 0.79 ms with 1 tile, 0.63 ms with 8-16, 0.72 ms with 32)
    const int tpb = (int)(tiles >= 8 * 768 ? 8 : (tiles >= 768 ? tiles / 768 : 1));
    const long long grid = ((tiles + tpb - 1) / tpb + 8 * TAIL_RUN - 1) / (8 * TAIL_RUN) * (8 * TAIL_RUN);
    if (grid > 0x7FFFFFFFLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((k_conv_tail3<CIN, TH>), dim3((unsigned)grid), dim3(256), lds, stream, a, tpb);
    return hipGetLastError();
}

// a.wp: [CIN/16][64 lanes][8] bf16 with row m = lane % 32 = tap*3 + co (rows 27..31 zero) and
// ci = 16*ks + 8*(lane/32) + e;  a.bias: 3 floats.
hipError_t rh_launch_conv_tail3(hipStream_t stream, int device, const conv_args& a, int cin)
{
    // tile height 7 for 64 channels: 0.57 ms against 0.61 with 8, 0.585 with 6, 0.59 with 5 rows on
    // 76 x 512 x 512 x 64 (9 x 34 patch pixels fill 10 MFMA column blocks with little padding)
    if (cin == 64) return launch_tail<64, 7>(stream, device, a);
    if (cin == 32) return launch_tail<32, 8>(stream, device, a);
    return hipErrorInvalidValue;
}

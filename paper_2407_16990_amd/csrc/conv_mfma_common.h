// Definitions shared by the MFMA convolution kernels (conv_mfma.hip, conv_mfma_duo.hip).
#pragma once
#include "rh_internal.h"

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(int)))) int i32x4;

struct conv_args {
    const __bf16* in;        // [N][H][W][CIN]
    const uint4* wp;         // packed weights of this layer
    const float* bias;       // packed order
    void* out;
    const __bf16* skip;      // same shape as out, or null
    const uint32_t* n_valid;
    int N, H, W;
    int relu, ps, n_chunks;  // bf16 output mode
    int cout_real, s_final;  // fp32 output mode
    int rev;                 // 1: walk the tiles from the last to the first (k_conv_mfma_duo)
    // box-masked mode (k_conv_mfma_duo): only the half tiles (8 rows x 32 pixels) listed are computed.
    // tile_list: RH_CELL_ENTRY(n, cy, tx) in any order, cy counting rows of 8; n_list: their number
    // (both dev); null: all tiles
    const uint32_t* tile_list;
    const uint32_t* n_list;
};

__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b)
{
    typedef __attribute__((__vector_size__(2 * sizeof(__bf16)))) __bf16 bf16x2;
    typedef __attribute__((__vector_size__(2 * sizeof(float)))) float f32x2;
    f32x2 v = {a, b};
    bf16x2 r = __builtin_convertvector(v, bf16x2);     // round to nearest even
    return *(uint32_t*)&r;
}

// ReLU of two packed bf16 values: a negative float has its sign bit set, i.e. is a negative
// 16-bit integer, and max(x, 0) on the integers leaves the others unchanged (-0 becomes +0).
// One packed instruction per pair, against two v_max_f32 per value for fmaxf on the fp32 inputs
// (the compiler adds a canonicalising max, also when the ReLU is written as a median of three).
__device__ __forceinline__ uint32_t relu_bf16x2(uint32_t u)
{
    typedef short s16x2 __attribute__((ext_vector_type(2)));
    const s16x2 z = {0, 0};
    const s16x2 r = __builtin_elementwise_max(*(const s16x2*)&u, z);
    return *(const uint32_t*)&r;
}

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load and store of the wave, which would expose the latency of the patch
// prefetch, the skip reads and the output stores once per tile.
__device__ __forceinline__ void lds_barrier() { asm volatile("s_waitcnt lgkmcnt(0)\n\ts_barrier" ::: "memory"); }

__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xFFFF0000u); }

#define RSRC_FLAGS 0x00020000            // raw buffer, 32-bit data format (gfx9 family)
#define OOB_OFF 0x80000000u              // beyond any descriptor used here (images are < 2 GiB)

// two-team kernel for the 64-channel bf16-output convs (conv_mfma_duo.hip)
hipError_t rh_launch_conv_duo(hipStream_t stream, int device, const conv_args& a, int grid, bool skip, bool relu);
// last conv with 3 output channels and no pixel shuffle (conv_tail.hip)
hipError_t rh_launch_conv_tail3(hipStream_t stream, int device, const conv_args& a, int cin);
// first conv 3 -> C on the matrix cores (conv_head.hip)
hipError_t rh_launch_head_mfma(hipStream_t stream, int C, const uint8_t* in, const uint4* wp, const float* bias, __bf16* out,
                               int N, int H, int W, int relu, const uint32_t* n_valid);
// upsampler + last conv of an EDSR-shaped net as one composed 5 x 5 conv (conv_fold.hip): t -> raw network output
// tile_list / n_list (dev, or null for all tiles): the 8 x 32 tiles to compute, as RH_CELL_ENTRY(n, ty, tx)
rh_status rh_launch_fold(rh_ctx* ctx, const __bf16* t, float* out, int N, int H, int W, const uint32_t* n_valid, int rev,
                         const uint32_t* tile_list, const uint32_t* n_list);

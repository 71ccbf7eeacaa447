// SR forward, fp32 path (Sec. 3.3.3): direct 3x3 convolutions on the vector ALUs.
// This is the high-precision path (configurations whose weights and activations are fp32);
// the throughput path is the bf16 MFMA one in conv_mfma.hip.
#include "rh_internal.h"

#define CO_T 8   // output channels per thread

// Thread = one pixel x CO_T output channels.  The output-channel block is uniform over the
// workgroup, so the weights are read through the scalar unit.  Input: f32 NHWC, or the u8
// image (then x/255 is taken here).  Epilogue: bias, optional ReLU, optional skip add,
// optional pixel shuffle by ps into out[N][H*ps][W*ps][Cout/ps^2].
__global__ __launch_bounds__(256) void k_conv3x3_f32(const void* __restrict__ in_, int in_u8,
                                                     const float* __restrict__ w, const float* __restrict__ bias,
                                                     float* out, const float* skip,
                                                     int H, int W, int Cin, int Cout, int relu, int ps,
                                                     const uint32_t* __restrict__ n_valid, int tiles_x)
{
    const int n = blockIdx.z;
    if (n_valid && (uint32_t)n >= *n_valid) return;
    const int tid = threadIdx.x, ty = blockIdx.x / tiles_x, tx = blockIdx.x - ty * tiles_x;
    const int x = tx * 16 + (tid & 15), y = ty * 16 + (tid >> 4);
    const int co0 = blockIdx.y * CO_T;
    if (x >= W || y >= H) return;
    float acc[CO_T];
    int cj[CO_T];
#pragma unroll
    for (int j = 0; j < CO_T; ++j) { cj[j] = min(co0 + j, Cout - 1); acc[j] = bias[cj[j]]; }
    const float* inf = (const float*)in_;
    const uint8_t* inb = (const uint8_t*)in_;
    for (int ky = 0; ky < 3; ++ky) {
        const int yy = y + ky - 1;
        if (yy < 0 || yy >= H) continue;
        for (int kx = 0; kx < 3; ++kx) {
            const int xx = x + kx - 1;
            if (xx < 0 || xx >= W) continue;
            const size_t pix = ((size_t)n * H + yy) * W + xx;
            const int tap = ky * 3 + kx;
            for (int ci = 0; ci < Cin; ++ci) {
                const float v = in_u8 ? __fdiv_rn((float)inb[pix * Cin + ci], 255.0f) : inf[pix * Cin + ci];
#pragma unroll
                for (int j = 0; j < CO_T; ++j) acc[j] = fmaf(w[((size_t)cj[j] * 9 + tap) * Cin + ci], v, acc[j]);
            }
        }
    }
    const int r2 = ps * ps, Co = Cout / r2;
#pragma unroll
    for (int j = 0; j < CO_T; ++j) {
        const int co = co0 + j;
        if (co >= Cout) break;
        float v = acc[j];
        if (relu) v = fmaxf(v, 0.0f);
        const int c = co / r2, sub = co - c * r2, si = sub / ps, sj = sub - si * ps;
        const size_t o = (((size_t)n * H * ps + (size_t)y * ps + si) * (W * ps) + (size_t)x * ps + sj) * Co + c;
        if (skip) v += skip[o];
        out[o] = v;
    }
}

static void conv(rh_ctx* ctx, const rh_layer& L, const void* in, int in_u8, float* out, const float* skip,
                 int N, int H, int W, int relu, int ps, const uint32_t* n_valid)
{
    const int tiles_x = (W + 15) / 16, tiles_y = (H + 15) / 16;
    hipLaunchKernelGGL(k_conv3x3_f32, dim3(tiles_x * tiles_y, (L.cout + CO_T - 1) / CO_T, N), dim3(256), 0,
                       ctx->stream, in, in_u8, ctx->w_f32 + L.w_off, ctx->w_f32 + L.b_off, out, skip, H, W, L.cin,
                       L.cout, relu, ps, n_valid, tiles_x);
}

rh_status rh_launch_enhance_fp32(rh_ctx* ctx, const uint8_t* in, int N, int H, int W, float* out,
                                 const uint32_t* n_valid)
{
    const rh_net_desc& d = ctx->cfg.net;
    const int C = d.channels, s = d.scale;
    const size_t lr = (size_t)N * H * W * C;
    size_t need = 3 * lr;
    size_t up1 = 0, up2 = 0;
    if (d.topology == RH_NET_EDSR) {
        const int r = (s == 4) ? 2 : s;
        up1 = lr * r * r; need += up1;
        if (s == 4) { up2 = up1 * 4; need += up2; }
    }
    rh_status st = rh_ensure_workspace(ctx, need * sizeof(float));
    if (st != RH_OK) return st;
    float* a = (float*)ctx->act; float* t = a + lr; float* h = t + lr; float* u1 = h + lr; float* u2 = u1 + up1;
    const std::vector<rh_layer>& L = ctx->layers;
    size_t li = 0;
    rh_prof_scope ps(ctx, RH_PROF_CONV, (uint32_t)L.size());     // all layers of the fp32 path count as one class
    // exact-border mode (a no-op otherwise): clear the out-of-frame part of the boxes in a layer's output
#define ZERO(buf, res) do { st = rh_zero_outside(ctx, (buf), C * (int)sizeof(float), (res), N, n_valid); if (st != RH_OK) return st; } while (0)
    if (d.topology == RH_NET_PLAIN) {
        conv(ctx, L[li++], in, 1, a, nullptr, N, H, W, 1, 1, n_valid); ZERO(a, 1);
        for (int l = 0; l < d.n_blocks - 2; ++l) { conv(ctx, L[li++], a, 0, t, nullptr, N, H, W, 1, 1, n_valid); ZERO(t, 1); float* sw = a; a = t; t = sw; }
        conv(ctx, L[li++], a, 0, out, nullptr, N, H, W, 0, s, n_valid);
    } else {
        conv(ctx, L[li++], in, 1, h, nullptr, N, H, W, 0, 1, n_valid); ZERO(h, 1);
        const float* x = h;                         // block input; the head output stays in h for EDSR
        for (int b = 0; b < d.n_blocks; ++b) {
            conv(ctx, L[li++], x, 0, t, nullptr, N, H, W, 1, 1, n_valid); ZERO(t, 1);
            // x + conv(t): for the first block the result goes to a so that h survives
            conv(ctx, L[li++], t, 0, a, x, N, H, W, 0, 1, n_valid); ZERO(a, 1);
            x = a;
        }
        if (d.topology == RH_NET_RES) {
            conv(ctx, L[li++], x, 0, out, nullptr, N, H, W, 0, s, n_valid);
        } else {
            conv(ctx, L[li++], x, 0, t, h, N, H, W, 0, 1, n_valid); ZERO(t, 1);         // body end + long skip
            const int r = (s == 4) ? 2 : s;
            conv(ctx, L[li++], t, 0, u1, nullptr, N, H, W, 0, r, n_valid); ZERO(u1, r);
            const float* last = u1; int hh = H * r, ww = W * r;
            if (s == 4) { conv(ctx, L[li++], u1, 0, u2, nullptr, N, hh, ww, 0, 2, n_valid); ZERO(u2, 2 * r); last = u2; hh *= 2; ww *= 2; }
            conv(ctx, L[li++], last, 0, out, nullptr, N, hh, ww, 0, 1, n_valid);
        }
    }
#undef ZERO
    RH_HIP(ctx, hipGetLastError());
    return RH_OK;
}

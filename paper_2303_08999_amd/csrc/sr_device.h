// Device-side helpers shared by every kernel of the library (gfx950 only).
//
// Stage 1 of the path (paper section II-B): separable cubic-convolution
// up-sampling.  Every kernel that needs an up-sampled value U[Y][X] goes through
// keys_weights() and dot4() below in the same order (vertical pass over four LR
// rows, then horizontal pass over four columns), so the fused kernels and the
// stand-alone up-sampler produce bit-identical U.
//
// The library is built with -ffp-contract=off: every fused multiply-add is
// written out with fmaf(), nothing is contracted behind our back.
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <stdint.h>

#include "../../include/sr_dict.h"

namespace srd {

// Kernel arguments common to the assembly kernels (passed by value).
struct AssembleArgs {
    const void*  lr;      // [N][C][h][w]
    const void*  coeff;   // [N][L][H][W]
    const float* dict;    // [L][k][k]
    void*        out;     // [N][C][H][W]
    int N, C, h, w, H, W, s, L;
    int xlast;            // matrix-core kernel: first column of the last tile column (set at launch)
    int n_fold;           // atoms folded: L (dense) or n_kept
    int io_f16;           // lr and out are fp16 (else fp32)
    int coeff_dtype;      // sr_dtype of the stored coefficients
    const unsigned char* index;   // list form only: atom numbers [N][T][H][W]; `coeff` then holds the values [N][T][H][W]
    int T;                // list form only: entries per pixel
    int pre_shuffle;      // coefficients are [N][L*s*s][h][w] (before the network's pixel-shuffle), else [N][L][H][W]
    int pixel_major;      // coefficients are [N][H][W][L] (a pixel's L coefficients side by side)
    int blocked;          // coefficients are stored in the blocked order (SR_COEFF_BLOCKED)
    int wb_ticks;         // matrix-core kernel (set at launch): period of the L2 write-back pacing in ticks of the constant clock, 0 = off
    int wb_flushers;      // ... and the workgroups 0 .. wb_flushers - 1 that ask for it: one per XCD of the device
    int logits;           // `coeff` holds logits: the coefficients are their per-pixel softmax over the atoms
    int   kept[SR_MAX_ATOMS];    // plane read for folded atom i (identity when dense)
    float gamma[SR_MAX_ATOMS];   // its scale (1 when dense)
};

struct BicubicArgs {
    const void* lr;
    void*       out;
    int NC, h, w, H, W, s;
};

__device__ __forceinline__ int clampi(int v, int lo, int hi) {
    return v < lo ? lo : (v > hi ? hi : v);
}

__device__ __forceinline__ float ld_as_float(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ld_as_float(const __half* p, size_t i) { return __half2float(p[i]); }
// fp8 e4m3 (OCP: bias 7, no infinities, largest 448) coefficient, one byte each;
// the conversion instruction widens exactly
struct f8e4m3 { unsigned char bits; };
__device__ __forceinline__ float ld_as_float(const f8e4m3* p, size_t i) {
    return __builtin_amdgcn_cvt_f32_fp8((int)p[i].bits, 0);
}
// bfloat16 coefficient, two bytes each: the upper half of a binary32
struct bf16raw { unsigned short bits; };
__device__ __forceinline__ float ld_as_float(const bf16raw* p, size_t i) {
    return __uint_as_float((unsigned)p[i].bits << 16);
}
// Logits form (coefficients = per-pixel softmax over the atoms of stored logits): the exponential of a logit z
// with nm = logit_shift(the pixel's largest logit), in fp32; every kernel rounds it to fp16 before use.
constexpr float LOG2E = 1.44269504088896340736f;
__device__ __forceinline__ float logit_shift(float m) { return -m * LOG2E; }
__device__ __forceinline__ float logit_exp(float z, float nm) { return __builtin_amdgcn_exp2f(fmaf(z, LOG2E, nm)); }
__device__ __forceinline__ void st_from_float(float* p, size_t i, float v) { p[i] = v; }
// fp32 -> fp16 with the fp32 value materialised first: the empty asm keeps the
// compiler from folding the producing fma and the narrowing into one
// mixed-precision instruction (a single rounding), so every kernel narrows the
// same fp32 value the same way.
__device__ __forceinline__ __half narrow_f16(float v) {
    asm volatile("" : "+v"(v));
    return __float2half_rn(v);
}
__device__ __forceinline__ void st_from_float(__half* p, size_t i, float v) { p[i] = narrow_f16(v); }

// Source position of HR index Y (0 <= Y) at integer scale s, half-pixel
// centres: source = (2Y + 1 - s) / (2s).  Returns floor(source); `m` receives
// the numerator of the fractional part over 2s (0 <= m < 2s).  Integer
// arithmetic only, so large coordinates lose nothing.
template <int S>
__device__ __forceinline__ int src_floor_s(int Y, int& m) {
    constexpr int two_s = 2 * S;
    const int num = 2 * Y + 1 - S + two_s;      // > 0 for Y >= 0
    const int q = num / two_s;                   // constant divisor
    m = num - q * two_s;
    return q - 1;
}
__device__ __forceinline__ int src_floor(int Y, int s, int& m) {
    switch (s) {                                 // wave-uniform branch
    case 2:  return src_floor_s<2>(Y, m);
    case 3:  return src_floor_s<3>(Y, m);
    default: return src_floor_s<4>(Y, m);
    }
}

// Keys cubic-convolution weights (a = -1/2) for taps floor-1 .. floor+2 at
// fractional offset t = m / (2s).  Exact in fp32 for s = 2 and s = 4.
__device__ __forceinline__ void keys_weights(int m, int s, float w[4]) {
    const float t = (float)m / (float)(2 * s);
    const float u0 = 1.0f + t, u1 = t, u2 = 1.0f - t, u3 = 2.0f - t;
    // 1 < |u| < 2 :  ((-1/2 u + 5/2) u - 4) u + 2
    w[0] = fmaf(fmaf(fmaf(-0.5f, u0, 2.5f), u0, -4.0f), u0, 2.0f);
    w[3] = fmaf(fmaf(fmaf(-0.5f, u3, 2.5f), u3, -4.0f), u3, 2.0f);
    // |u| <= 1    :  (3/2 u - 5/2) u^2 + 1
    w[1] = fmaf(fmaf(1.5f, u1, -2.5f), u1 * u1, 1.0f);
    w[2] = fmaf(fmaf(1.5f, u2, -2.5f), u2 * u2, 1.0f);
}

__device__ __forceinline__ float dot4(const float w[4], float a, float b, float c, float d) {
    float r = w[0] * a;
    r = fmaf(w[1], b, r);
    r = fmaf(w[2], c, r);
    r = fmaf(w[3], d, r);
    return r;
}

// ---------------------------------------------------------------------------
// Cooperative production of an up-sampled tile in LDS.
//
// The tile covers HR rows Y0-R .. Y0-R+UH-1 and columns X0-R .. X0-R+UW-1;
// coordinates outside the image are clamped BEFORE the interpolator is
// evaluated (the up-sampled image is replicate-padded).  Phases, the caller
// puts a workgroup barrier between them:
//   build_taps (x and y) + LR footprint -> lrT [MAXLRY][MAXLRX]   (clamped reads)
//   vertical pass  : V[yy][rx] = dot4(wy[yy], lrT[yb[yy] .. +3][rx])
//   horizontal pass: U[yy][xx] = dot4(wx[xx], V[yy][xb[xx] .. +3])
// Vertical first: the intermediate is only as wide as the LR footprint.  Every
// kernel of the library evaluates stage 1 in this order, so their up-sampled
// values agree bit for bit.  MAXLR* must be >= ceil((extent-1)/s) + 4 for the
// smallest scale the kernel is launched with.
// ---------------------------------------------------------------------------
struct TileOrigin {
    int ly0, lx0;   // LR coordinate of lrT[0][0] (may be negative: reads are clamped)
    int nly, nlx;   // LR rows / columns the tile really needs (<= MAXLRY / MAXLRX)
};

__device__ __forceinline__ TileOrigin tile_origin(int Y0, int X0, int R, int UH, int UW, int H, int W, int s) {
    int m;
    TileOrigin o;
    o.ly0 = src_floor(clampi(Y0 - R, 0, H - 1), s, m) - 1;
    o.lx0 = src_floor(clampi(X0 - R, 0, W - 1), s, m) - 1;
    o.nly = src_floor(clampi(Y0 - R + UH - 1, 0, H - 1), s, m) + 2 - o.ly0 + 1;
    o.nlx = src_floor(clampi(X0 - R + UW - 1, 0, W - 1), s, m) + 2 - o.lx0 + 1;
    return o;
}

// Per-coordinate interpolation taps of one tile axis: weights and the index of
// the first of the four source rows/columns inside the LDS footprint.
template <int N, int MAXLR, int NT>
__device__ __forceinline__ void build_taps(int origin, int R, int limit, int s, int l0,
                                           float4* __restrict__ wtab, int* __restrict__ btab, int tid) {
    for (int i = tid; i < N; i += NT) {
        int m;
        const int f = src_floor(clampi(origin - R + i, 0, limit - 1), s, m);
        float wt[4];
        keys_weights(m, s, wt);
        wtab[i] = make_float4(wt[0], wt[1], wt[2], wt[3]);
        btab[i] = clampi(f - 1 - l0, 0, MAXLR - 4);   // the clamp never moves a needed tap
    }
}

template <typename TIO, int MAXLRY, int MAXLRX, int NT>
__device__ __forceinline__ void load_lr_tile(const TIO* __restrict__ plane, int h, int w,
                                             TileOrigin o, float* __restrict__ lrT, int tid) {
    for (int idx = tid; idx < MAXLRY * MAXLRX; idx += NT) {
        const int ry = idx / MAXLRX, rx = idx - ry * MAXLRX;
        const int yy = clampi(o.ly0 + ry, 0, h - 1);
        const int xx = clampi(o.lx0 + rx, 0, w - 1);
        lrT[idx] = ld_as_float(plane, (size_t)yy * w + xx);
    }
}

// vertical pass, one element per step: V[yy][rx], pitch MAXLRX
template <int MAXLRX, int UH, int NT>
__device__ __forceinline__ void vpass(const float* __restrict__ lrT, float* __restrict__ V,
                                      const float4* __restrict__ yw, const int* __restrict__ yb, int tid) {
    for (int idx = tid; idx < UH * MAXLRX; idx += NT) {
        const int yy = idx / MAXLRX, rx = idx - yy * MAXLRX;
        const float4 w4 = yw[yy];
        const float wt[4] = {w4.x, w4.y, w4.z, w4.w};
        const float* p = lrT + yb[yy] * MAXLRX + rx;
        V[idx] = dot4(wt, p[0], p[MAXLRX], p[2 * MAXLRX], p[3 * MAXLRX]);
    }
}

// horizontal pass, one element per step
template <int MAXLRX, int UW, int UH, int NT, typename Store>
__device__ __forceinline__ void hpass(const float* __restrict__ V,
                                      const float4* __restrict__ xw, const int* __restrict__ xb,
                                      int tid, Store store) {
    for (int idx = tid; idx < UH * UW; idx += NT) {
        const int yy = idx / UW, xx = idx - yy * UW;
        const float4 w4 = xw[xx];
        const float wt[4] = {w4.x, w4.y, w4.z, w4.w};
        const float* p = V + yy * MAXLRX + xb[xx];
        store(yy, xx, dot4(wt, p[0], p[1], p[2], p[3]));
    }
}

}  // namespace srd

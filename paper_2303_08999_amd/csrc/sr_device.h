// Device-side helpers shared by every kernel of the library (gfx950 only).
//
// Stage 1 of the path (paper section II-B): separable cubic-convolution
// up-sampling.  Every kernel that needs an up-sampled value U[Y][X] goes through
// keys_weights() and dot4() below in the same order (horizontal pass over four
// LR columns, then vertical pass over four LR rows), so the fused kernels and
// the stand-alone up-sampler produce bit-identical U.
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
    int n_fold;           // atoms folded: L (dense) or n_kept
    int io_f16;           // lr and out are fp16 (else fp32)
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
//   hpass : four-tap horizontal pass    -> hbuf [nly][UW]
//   vpass : four-tap vertical pass      -> U via store(yy, xx, value)
// MAXLR* must be >= ceil((extent-1)/s) + 4 for the smallest scale (2).
// ---------------------------------------------------------------------------
struct TileOrigin {
    int ly0, lx0;   // LR coordinate of lrT[0][0] (may be negative: reads are clamped)
    int nly;        // LR rows the tile really needs (<= MAXLRY)
};

__device__ __forceinline__ TileOrigin tile_origin(int Y0, int X0, int R, int UH, int H, int W, int s) {
    int m;
    TileOrigin o;
    o.ly0 = src_floor(clampi(Y0 - R, 0, H - 1), s, m) - 1;
    o.lx0 = src_floor(clampi(X0 - R, 0, W - 1), s, m) - 1;
    o.nly = src_floor(clampi(Y0 - R + UH - 1, 0, H - 1), s, m) + 2 - o.ly0 + 1;
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

template <int MAXLRX, int UW, int NT>
__device__ __forceinline__ void hpass(const float* __restrict__ lrT, float* __restrict__ hbuf,
                                      const float4* __restrict__ xw, const int* __restrict__ xb,
                                      int nly, int tid) {
    for (int idx = tid; idx < nly * UW; idx += NT) {
        const int ry = idx / UW, xx = idx - ry * UW;
        const float4 w4 = xw[xx];
        const float wt[4] = {w4.x, w4.y, w4.z, w4.w};
        const float* p = lrT + ry * MAXLRX + xb[xx];
        hbuf[idx] = dot4(wt, p[0], p[1], p[2], p[3]);
    }
}

template <int UW, int UH, int NT, typename Store>
__device__ __forceinline__ void vpass(const float* __restrict__ hbuf,
                                      const float4* __restrict__ yw, const int* __restrict__ yb,
                                      int tid, Store store) {
    for (int idx = tid; idx < UH * UW; idx += NT) {
        const int yy = idx / UW, xx = idx - yy * UW;
        const float4 w4 = yw[yy];
        const float wt[4] = {w4.x, w4.y, w4.z, w4.w};
        const float* p = hbuf + yb[yy] * UW + xx;
        store(yy, xx, dot4(wt, p[0], p[UW], p[2 * UW], p[3 * UW]));
    }
}

// Column-per-thread forms of the two passes (used by the matrix-core kernel):
// a thread owns one (channel, column) and walks the rows, so the tap weights of
// the horizontal pass are loaded once per thread and the vertical pass keeps a
// sliding window of four values in registers.  Same dot4() per element as above.
template <int C, int MAXLRY, int MAXLRX, int UW, int NT>
__device__ __forceinline__ void hpass_cols(const float* __restrict__ lrT, float* __restrict__ hbuf,
                                           const float4* __restrict__ xw, const int* __restrict__ xb,
                                           int nly, int tid) {
    for (int col = tid; col < C * UW; col += NT) {
        const int c = col / UW, xx = col - c * UW;
        const float4 w4 = xw[xx];
        const float wt[4] = {w4.x, w4.y, w4.z, w4.w};
        const float* src = lrT + c * MAXLRY * MAXLRX + xb[xx];
        float* dst = hbuf + c * MAXLRY * UW + xx;
        for (int ry = 0; ry < nly; ++ry) {
            const float* p = src + ry * MAXLRX;
            dst[ry * UW] = dot4(wt, p[0], p[1], p[2], p[3]);
        }
    }
}

template <int C, int MAXLRY, int UW, int UH, int NT, typename Store>
__device__ __forceinline__ void vpass_cols(const float* __restrict__ hbuf,
                                           const float4* __restrict__ yw, const int* __restrict__ yb,
                                           int tid, Store store) {
    for (int col = tid; col < C * UW; col += NT) {
        const int c = col / UW, xx = col - c * UW;
        const float* src = hbuf + c * MAXLRY * UW + xx;
        int bcur = __builtin_amdgcn_readfirstlane(yb[0]);
        float h0 = src[bcur * UW], h1 = src[(bcur + 1) * UW], h2 = src[(bcur + 2) * UW], h3 = src[(bcur + 3) * UW];
#pragma unroll
        for (int yy = 0; yy < UH; ++yy) {
            const int b = __builtin_amdgcn_readfirstlane(yb[yy]);   // the same for every thread
            if (b == bcur + 1) {
                h0 = h1; h1 = h2; h2 = h3; h3 = src[(b + 3) * UW];
            } else if (b != bcur) {
                h0 = src[b * UW]; h1 = src[(b + 1) * UW]; h2 = src[(b + 2) * UW]; h3 = src[(b + 3) * UW];
            }
            bcur = b;
            const float4 w4 = yw[yy];
            const float wt[4] = {w4.x, w4.y, w4.z, w4.w};
            store(c, yy, xx, dot4(wt, h0, h1, h2, h3));
        }
    }
}

}  // namespace srd

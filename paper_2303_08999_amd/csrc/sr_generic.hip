// Generic fp32 vector-ALU kernels: every supported (dtype, k, L, C, scale, size)
// combination, including odd widths and kept-atom lists.  One thread per HR
// pixel; the fold F_i = Phi_i D (paper Eq. 2, stage 3) is kept in registers,
// the up-sampled patch tile (stage 1) lives in LDS, the filtering
// y_i = F_i B_i^T (stage 4) reads it from there.  The matrices F and B of
// Eq. 3 are never written to memory.
//
// This kernel is bound by the fp32 ALUs (L*k^2 multiply-adds per pixel), not by
// HBM; the matrix-core kernel (sr_mfma_kernel.h) is the fast path wherever it
// qualifies.
#include "sr_device.h"
#include "sr_launch.h"

namespace srd {

constexpr int GTW = 64;   // tile width  (HR pixels) = one wavefront per row
constexpr int GTH = 4;    // tile height (HR pixels)
constexpr int GNT = GTW * GTH;

template <typename TC, typename TIO, int K>
__global__ __launch_bounds__(GNT) void k_assemble_generic(const AssembleArgs a) {
    constexpr int KK = K * K;
    constexpr int R = (K - 1) / 2;
    constexpr int UW = GTW + K - 1;
    constexpr int UH = GTH + K - 1;
    constexpr int MAXLRY = (UH - 1) / 2 + 5;   // scale >= 2
    constexpr int MAXLRX = (UW - 1) / 2 + 5;

    __shared__ float lrT[MAXLRY * MAXLRX];
    __shared__ float V[UH * MAXLRX];
    __shared__ float U[UH * UW];
    __shared__ float4 xw[UW], yw[UH];
    __shared__ int xb[UW], yb[UH];

    const int tid = threadIdx.x;
    const int tx = tid % GTW, ty = tid / GTW;
    const int X0 = blockIdx.x * GTW, Y0 = blockIdx.y * GTH, n = blockIdx.z;
    const int X = X0 + tx, Y = Y0 + ty;
    const bool valid = X < a.W && Y < a.H;
    const size_t plane = (size_t)a.H * a.W;

    // ---- stage 3: F = Phi_i D, all k^2 taps in registers -------------------
    float F[KK];
    float esum = 0.0f;                                      // logits form: sum of the pixel's exponentials
#pragma unroll
    for (int t = 0; t < KK; ++t) F[t] = 0.0f;
    if (valid) {
        // where this pixel's coefficient lies within an atom's H*W elements: row-major HR plane, or (before the
        // network's pixel-shuffle) s*s LR planes, the one for this pixel's row and column modulo s
        const size_t within = a.pre_shuffle
            ? (size_t)((Y % a.s) * a.s + X % a.s) * ((size_t)a.h * a.w) + (size_t)(Y / a.s) * a.w + X / a.s
            : (size_t)Y * a.W + X;
        // ... or, pixel-major, the pixel's L coefficients side by side
        const size_t astride = a.pixel_major ? (size_t)1 : plane;
        // ... or blocked: units of 128 pixels, four slots (pixel 4 j + q is slot q, column j) of 32 L elements, pieces of
        // 16 atoms [half][j][8] and a last piece [half][j][4] (see SR_COEFF_BLOCKED); atom l of this pixel is at
        // blk_slot + blk_atom(l)
        const size_t blk_slot = (((size_t)Y * (a.W / 128) + X / 128) * 4 + X % 4) * ((size_t)32 * a.L);
        const int blk_j = (X % 128) / 4, blk_full = a.L / 16;
        auto blk_atom = [&](int l) -> size_t {
            if (l < 16 * blk_full) return (size_t)(l / 16) * 512 + (size_t)((l % 16) / 8) * 256 + (size_t)blk_j * 8 + l % 8;
            const int t = l - 16 * blk_full;
            return (size_t)blk_full * 512 + (size_t)(t / 4) * 128 + (size_t)blk_j * 4 + t % 4;
        };
        const TC* cbase = (const TC*)a.coeff + (size_t)n * a.L * plane + (a.blocked ? blk_slot : a.pixel_major ? within * a.L : within);
        auto coff = [&](int l) -> size_t { return a.blocked ? blk_atom(l) : (size_t)l * astride; };
        // eight atoms at a time: their coefficient loads are in flight together
        constexpr int NB = 8;
        // logits instead of coefficients: a first pass over the pixel's planes for the largest logit
        float nm = 0.0f;
        if (a.logits) {
            float m = ld_as_float(cbase, coff(0));
            for (int i0 = 0; i0 < a.n_fold; i0 += NB) {
                float z[NB];
#pragma unroll
                for (int b = 0; b < NB; ++b) z[b] = ld_as_float(cbase, coff(i0 + b < a.n_fold ? i0 + b : a.n_fold - 1));
#pragma unroll
                for (int b = 0; b < NB; ++b) m = fmaxf(m, z[b]);
            }
            nm = logit_shift(m);
        }
        for (int i0 = 0; i0 < a.n_fold; i0 += NB) {
            float phi[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
                const int i = i0 + b < a.n_fold ? i0 + b : a.n_fold - 1;      // past the end: re-read, unused
                phi[b] = ld_as_float(cbase, coff(a.kept[i])) * a.gamma[i];
                if (a.logits) {                             // (no kept list, gamma = 1): exponential, rounded to fp16
                    phi[b] = __half2float(__float2half_rn(logit_exp(phi[b], nm)));
                    if (i0 + b < a.n_fold) esum += phi[b];
                }
            }
#pragma unroll
            for (int b = 0; b < NB; ++b)
                if (i0 + b < a.n_fold) {                    // wave-uniform
                    const float* d = a.dict + (size_t)a.kept[i0 + b] * KK;   // wave-uniform: scalar loads
#pragma unroll
                    for (int t = 0; t < KK; ++t) F[t] = fmaf(phi[b], d[t], F[t]);
                }
        }
    }

    // ---- stages 1 + 4, one channel at a time -------------------------------
    const TileOrigin o = tile_origin(Y0, X0, R, UH, UW, a.H, a.W, a.s);
    build_taps<UW, MAXLRX, GNT>(X0, R, a.W, a.s, o.lx0, xw, xb, tid);
    build_taps<UH, MAXLRY, GNT>(Y0, R, a.H, a.s, o.ly0, yw, yb, tid);
    for (int c = 0; c < a.C; ++c) {
        const TIO* lrp = (const TIO*)a.lr + ((size_t)n * a.C + c) * (size_t)a.h * a.w;
        load_lr_tile<TIO, MAXLRY, MAXLRX, GNT>(lrp, a.h, a.w, o, lrT, tid);
        __syncthreads();
        vpass<MAXLRX, UH, GNT>(lrT, V, yw, yb, tid);
        __syncthreads();
        hpass<MAXLRX, UW, UH, GNT>(V, xw, xb, tid, [&](int yy, int xx, float v) { U[yy * UW + xx] = v; });
        __syncthreads();
        if (valid) {
            float acc = 0.0f;
#pragma unroll
            for (int dy = 0; dy < K; ++dy)
#pragma unroll
                for (int dx = 0; dx < K; ++dx)
                    acc = fmaf(F[dy * K + dx], U[(ty + dy) * UW + tx + dx], acc);
            if (a.logits) acc = acc * (1.0f / esum);
            st_from_float((TIO*)a.out, ((size_t)n * a.C + c) * plane + (size_t)Y * a.W + X, acc);
        }
        // The next channel's lrT/V writes do not touch U; two barriers separate
        // this read of U from the next horizontal pass.
    }
}

// Stage 1 alone, same arithmetic as the tiles (vertical pass over four LR rows, then
// horizontal pass over four columns), so the values agree bit for bit with the U
// the fused kernels form.  A workgroup produces 256 x 16 pixels: it loads their LR
// footprint (at most 12 rows x 132 columns) into LDS once, forms the vertical pass
// of the 16 rows there, and each thread then produces four consecutive pixels of
// four rows, each group stored with one 16-byte (fp16: 8-byte) store when the rows
// keep that alignment.
// (Before: every thread gathered its own 24 LR pixels from global memory; the 4K
// frame took 50 us against 16 us for the bare 99.5 MB write.)
template <typename TI, typename TO>
__global__ __launch_bounds__(256) void k_bicubic(const BicubicArgs a) {
    constexpr int PXT = 4;                // pixels of a thread in a row
    constexpr int BW = 256, BH = 16;      // pixels of a workgroup
    constexpr int MAXC = BW / 2 + 4, MAXR = BH / 2 + 4;     // LR footprint at the smallest scale, 2
    constexpr int MAXS = 4;               // largest scale
    __shared__ float lrT[MAXR][MAXC];
    __shared__ float V[BH][MAXC];
    __shared__ float4 wyT[BH], wxT[2 * MAXS];    // weights of the workgroup's rows; weights by phase m
    __shared__ int rbT[BH];                      // first footprint row of each row's four taps
    const int tid = threadIdx.x;
    const int Xb = blockIdx.x * BW, Yb = blockIdx.y * BH, nc = blockIdx.z;
    const TI* p = (const TI*)a.lr + (size_t)nc * a.h * a.w;
    int m;
    const int c0 = src_floor(Xb, a.s, m) - 1;                                   // first LR column and row (may be -1 or -2: clamped)
    const int r0 = src_floor(Yb, a.s, m) - 1;
    const int ncol = src_floor(clampi(Xb + BW - 1, 0, a.W - 1), a.s, m) + 2 - c0 + 1;
    const int nrow = src_floor(clampi(Yb + BH - 1, 0, a.H - 1), a.s, m) + 2 - r0 + 1;
    // e / ncol for e < 2^14 without a division per element (4 <= ncol <= 132: exact)
    const unsigned inv = ((1u << 22) + ncol - 1) / ncol;
    for (int e = tid; e < nrow * ncol; e += 256) {
        const int r = (int)(((unsigned)e * inv) >> 22), c = e - r * ncol;
        lrT[r][c] = ld_as_float(p, (size_t)clampi(r0 + r, 0, a.h - 1) * a.w + clampi(c0 + c, 0, a.w - 1));
    }
    if (tid < BH) {
        int my;
        rbT[tid] = src_floor(clampi(Yb + tid, 0, a.H - 1), a.s, my) - 1 - r0;
        float w[4];
        keys_weights(my, a.s, w);
        wyT[tid] = make_float4(w[0], w[1], w[2], w[3]);
    } else if (tid >= 64 && tid < 64 + 2 * a.s) {
        float w[4];
        keys_weights(tid - 64, a.s, w);
        wxT[tid - 64] = make_float4(w[0], w[1], w[2], w[3]);
    }
    __syncthreads();
    for (int e = tid; e < BH * ncol; e += 256) {
        const int r = (int)(((unsigned)e * inv) >> 22), c = e - r * ncol;
        const int rb = rbT[r];
        const float4 w4 = wyT[r];
        const float wy[4] = {w4.x, w4.y, w4.z, w4.w};
        V[r][c] = dot4(wy, lrT[rb][c], lrT[rb + 1][c], lrT[rb + 2][c], lrT[rb + 3][c]);
    }
    __syncthreads();
    const int X0 = Xb + (tid % 64) * PXT;
    if (X0 >= a.W) return;
    // Each pixel reads its own four vertical-pass columns from LDS.  (Sharing the six
    // columns of the group in registers needs a select per tap, which the compiler
    // turns into divergent branches: measured 2 x slower.)
    int col[PXT];
    float wx[PXT][4];
#pragma unroll
    for (int q = 0; q < PXT; ++q) {
        int mx;
        col[q] = src_floor(X0 + q < a.W ? X0 + q : a.W - 1, a.s, mx) - 1 - c0;      // .. + 3 < ncol
        const float4 w4 = wxT[mx];
        wx[q][0] = w4.x; wx[q][1] = w4.y; wx[q][2] = w4.z; wx[q][3] = w4.w;
    }
    const bool vec = (a.W & 3) == 0 && ((uintptr_t)a.out & 15) == 0;    // whole groups, 16-byte aligned rows
    const int rt = tid / 64;
#pragma unroll
    for (int i = 0; i < BH / 4; ++i) {
        const int r = rt + 4 * i;
        if (Yb + r >= a.H) break;
        float res[PXT];
#pragma unroll
        for (int q = 0; q < PXT; ++q) {
            const float* v = &V[r][col[q]];
            res[q] = dot4(wx[q], v[0], v[1], v[2], v[3]);
        }
        TO* dst = (TO*)a.out + ((size_t)nc * a.H + Yb + r) * a.W + X0;
        if (vec) {
            if constexpr (sizeof(TO) == 4) {
                *(float4*)dst = make_float4(res[0], res[1], res[2], res[3]);
            } else {
                union { __half h[4]; uint2 u; } pk;
#pragma unroll
                for (int q = 0; q < PXT; ++q) pk.h[q] = narrow_f16(res[q]);
                *(uint2*)dst = pk.u;
            }
        } else {
#pragma unroll
            for (int q = 0; q < PXT; ++q)
                if (X0 + q < a.W) st_from_float(dst, q, res[q]);
        }
    }
}

template <typename TC, typename TIO>
static hipError_t launch_generic_k(const AssembleArgs& a, int k, hipStream_t st) {
    const dim3 grid((a.W + GTW - 1) / GTW, (a.H + GTH - 1) / GTH, a.N);
    switch (k) {
    case 3: hipLaunchKernelGGL((k_assemble_generic<TC, TIO, 3>), grid, dim3(GNT), 0, st, a); break;
    case 5: hipLaunchKernelGGL((k_assemble_generic<TC, TIO, 5>), grid, dim3(GNT), 0, st, a); break;
    case 7: hipLaunchKernelGGL((k_assemble_generic<TC, TIO, 7>), grid, dim3(GNT), 0, st, a); break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

hipError_t launch_generic(const AssembleArgs& a, int k, bool io_f16, hipStream_t st) {
    if (a.coeff_dtype == SR_F16)
        return io_f16 ? launch_generic_k<__half, __half>(a, k, st) : launch_generic_k<__half, float>(a, k, st);
    if (a.coeff_dtype == SR_F8E4M3)
        return io_f16 ? launch_generic_k<f8e4m3, __half>(a, k, st) : launch_generic_k<f8e4m3, float>(a, k, st);
    if (a.coeff_dtype == SR_BF16)
        return io_f16 ? launch_generic_k<bf16raw, __half>(a, k, st) : launch_generic_k<bf16raw, float>(a, k, st);
    return io_f16 ? launch_generic_k<float, __half>(a, k, st) : launch_generic_k<float, float>(a, k, st);
}

hipError_t launch_bicubic(const BicubicArgs& a, bool in_f16, bool out_f16, hipStream_t st) {
    const dim3 grid((a.W + 255) / 256, (a.H + 15) / 16, a.NC);
    if (in_f16) {
        if (out_f16) hipLaunchKernelGGL((k_bicubic<__half, __half>), grid, dim3(256), 0, st, a);
        else         hipLaunchKernelGGL((k_bicubic<__half, float>), grid, dim3(256), 0, st, a);
    } else {
        if (out_f16) hipLaunchKernelGGL((k_bicubic<float, __half>), grid, dim3(256), 0, st, a);
        else         hipLaunchKernelGGL((k_bicubic<float, float>), grid, dim3(256), 0, st, a);
    }
    return hipGetLastError();
}

}  // namespace srd

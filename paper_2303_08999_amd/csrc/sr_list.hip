// Coefficients as per-pixel lists: for every HR pixel T entries (atom index, value) instead of L
// dense planes.  An EXTENSION beyond the paper, which selects atoms once for the whole model
// (section III-A); it follows the paper's own argument that what the fold skips should not be
// loaded (section II-A, Eq. 4): 3 T bytes per pixel instead of 2 L.  Computed is Eq. 2 with the
// listed terms only, F_i = sum_t value[t][i] D[index[t][i]], then y_i = F_i B_i^T as everywhere.
//
// A thread owns four consecutive pixels of a row and reads, per entry, their four indices and
// four values; the dictionary sits in LDS with rows padded to whole 16-byte groups and every
// entry gathers its atom's row from there; stage 1 and stage 4 are the generic kernel's
// (sr_generic.hip), on a 256 x 4 tile.  Bound: the LDS gathers (T * k^2 * 4 bytes per pixel),
// not HBM.  This kernel takes every supported case; 5x5 atoms, three channels and fp16 values
// go to the matrix-core kernel instead (CT_LIST8, CT_LIST16 in sr_mfma_kernel.h), which scatters
// the lists into the dense form's operands and is more than twice as fast.
#include <stdint.h>

#include <string.h>

#include "sr_launch.h"

namespace srd {

struct ListArgs {
    const void* lr;                  // [N][C][h][w]
    const unsigned char* index;      // [N][T][H][W]
    const void* value;               // [N][T][H][W]
    const float* dict;               // [L][k][k]
    void* out;                       // [N][C][H][W]
    int N, C, h, w, H, W, s, L, T;
};

namespace {

constexpr int LTW = 256, LTH = 4, LNT = 256, LPX = 4;     // tile, threads, pixels per thread

template <typename TV, typename TIO, int K>
__global__ __launch_bounds__(LNT) void k_assemble_list(const ListArgs a) {
    constexpr int KK = K * K, KKP = (KK + 3) / 4 * 4, R = (K - 1) / 2;
    constexpr int UW = LTW + K - 1, UH = LTH + K - 1;
    constexpr int MAXLRY = (UH - 1) / 2 + 5, MAXLRX = (UW - 1) / 2 + 5;     // scale >= 2
    extern __shared__ float4 Dl[];                    // [L][KKP / 4]: the dictionary, rows padded with zeros
    __shared__ float lrT[MAXLRY * MAXLRX];
    __shared__ float V[UH * MAXLRX];
    __shared__ float U[UH * UW];
    __shared__ float4 xw[UW], yw[UH];
    __shared__ int xb[UW], yb[UH];

    const int tid = threadIdx.x;
    const int tx = tid % 64, ty = tid / 64;
    const int X0 = blockIdx.x * LTW, Y0 = blockIdx.y * LTH, n = blockIdx.z;
    const int X = X0 + LPX * tx, Y = Y0 + ty;
    const size_t plane = (size_t)a.H * a.W;

    for (int e = tid; e < a.L * KKP; e += LNT) {
        const int l = e / KKP, j = e - l * KKP;
        ((float*)Dl)[e] = j < KK ? a.dict[(size_t)l * KK + j] : 0.0f;
    }
    __syncthreads();

    // ---- stage 3: F = sum over the listed entries, all k^2 taps of four pixels in registers
    float F[LPX][KKP];
#pragma unroll
    for (int q = 0; q < LPX; ++q)
#pragma unroll
        for (int t = 0; t < KKP; ++t) F[q][t] = 0.0f;
    if (Y < a.H && X < a.W) {
        const size_t at0 = (size_t)n * a.T * plane + (size_t)Y * a.W + X;
        const bool whole = X + LPX <= a.W;            // all four pixels inside the row
        const unsigned lmax = (unsigned)a.L - 1u;
        for (int t = 0; t < a.T; ++t) {
            const size_t at = at0 + (size_t)t * plane;
            unsigned idx[LPX];
            float val[LPX];
#pragma unroll
            for (int q = 0; q < LPX; ++q) {
                const bool in = whole || X + q < a.W;
                idx[q] = in ? (unsigned)a.index[at + q] : 0u;
                val[q] = in ? ld_as_float((const TV*)a.value, at + q) : 0.0f;
                idx[q] = idx[q] < lmax ? idx[q] : lmax;       // an index not below L never reads outside the table
            }
#pragma unroll
            for (int q = 0; q < LPX; ++q) {
                const float4* d = Dl + idx[q] * (KKP / 4);
#pragma unroll
                for (int g = 0; g < KKP / 4; ++g) {
                    const float4 dd = d[g];
                    F[q][4 * g + 0] = fmaf(val[q], dd.x, F[q][4 * g + 0]);
                    F[q][4 * g + 1] = fmaf(val[q], dd.y, F[q][4 * g + 1]);
                    F[q][4 * g + 2] = fmaf(val[q], dd.z, F[q][4 * g + 2]);
                    F[q][4 * g + 3] = fmaf(val[q], dd.w, F[q][4 * g + 3]);
                }
            }
        }
    }

    // ---- stages 1 + 4, one channel at a time (the generic kernel's passes)
    const TileOrigin o = tile_origin(Y0, X0, R, UH, UW, a.H, a.W, a.s);
    build_taps<UW, MAXLRX, LNT>(X0, R, a.W, a.s, o.lx0, xw, xb, tid);
    build_taps<UH, MAXLRY, LNT>(Y0, R, a.H, a.s, o.ly0, yw, yb, tid);
    for (int c = 0; c < a.C; ++c) {
        const TIO* lrp = (const TIO*)a.lr + ((size_t)n * a.C + c) * (size_t)a.h * a.w;
        load_lr_tile<TIO, MAXLRY, MAXLRX, LNT>(lrp, a.h, a.w, o, lrT, tid);
        __syncthreads();
        vpass<MAXLRX, UH, LNT>(lrT, V, yw, yb, tid);
        __syncthreads();
        hpass<MAXLRX, UW, UH, LNT>(V, xw, xb, tid, [&](int yy, int xx, float v) { U[yy * UW + xx] = v; });
        __syncthreads();
        if (Y < a.H && X < a.W) {
            float acc[LPX] = {0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int dy = 0; dy < K; ++dy) {
                float row[LPX + K - 1];
#pragma unroll
                for (int i = 0; i < LPX + K - 1; ++i) row[i] = U[(ty + dy) * UW + LPX * tx + i];
#pragma unroll
                for (int q = 0; q < LPX; ++q)
#pragma unroll
                    for (int dx = 0; dx < K; ++dx) acc[q] = fmaf(F[q][dy * K + dx], row[q + dx], acc[q]);
            }
            const size_t o0 = ((size_t)n * a.C + c) * plane + (size_t)Y * a.W + X;
#pragma unroll
            for (int q = 0; q < LPX; ++q)
                if (X + q < a.W) st_from_float((TIO*)a.out, o0 + q, acc[q]);
        }
    }
}

size_t esize(sr_dtype d) { return d == SR_F32 ? 4 : 2; }

bool overlap(const void* p, size_t np, const void* q, size_t nq) {
    const uintptr_t a0 = (uintptr_t)p, b0 = (uintptr_t)q;
    return a0 < b0 + nq && b0 < a0 + np;
}

template <typename TV, typename TIO>
hipError_t launch_list(const ListArgs& a, int k, hipStream_t st) {
    const dim3 grid((a.W + LTW - 1) / LTW, (a.H + LTH - 1) / LTH, a.N);
    const int kkp = (k * k + 3) / 4 * 4;
    const size_t lds = (size_t)a.L * kkp * sizeof(float);
    hipError_t e = hipSuccess;
    switch (k) {
    case 3: hipLaunchKernelGGL((k_assemble_list<TV, TIO, 3>), grid, dim3(LNT), lds, st, a); break;
    case 5: hipLaunchKernelGGL((k_assemble_list<TV, TIO, 5>), grid, dim3(LNT), lds, st, a); break;
    case 7:
        if (lds > 48 * 1024)
            e = hipFuncSetAttribute((const void*)k_assemble_list<TV, TIO, 7>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL((k_assemble_list<TV, TIO, 7>), grid, dim3(LNT), lds, st, a);
        break;
    default: return hipErrorInvalidValue;
    }
    return hipGetLastError();
}

}  // namespace
}  // namespace srd

using namespace srd;

static int assemble_list(const sr_tensor* lr, const sr_tensor* index, const sr_tensor* value, const sr_tensor* dict,
                         int L, int k, int scale, int channels, int entries, sr_tensor* out, void* stream, int force_kernel) {
    if (!lr || !index || !value || !dict || !out) return SR_ERR_NULL;
    if ((lr->dtype != SR_F32 && lr->dtype != SR_F16) || out->dtype != lr->dtype || index->dtype != SR_U8 ||
        (value->dtype != SR_F32 && value->dtype != SR_F16) || dict->dtype != SR_F32) return SR_ERR_UNSUPPORTED;
    for (const sr_tensor* t : {lr, index, value, dict, (const sr_tensor*)out})
        if (t->n < 0 || t->c < 0 || t->h < 0 || t->w < 0) return SR_ERR_SHAPE;
    if ((k != 3 && k != 5 && k != 7) || scale < 2 || scale > 4 || L < 1 || L > SR_MAX_ATOMS || channels < 1 ||
        channels > SR_MAX_CHANNELS || entries < 1 || entries > SR_MAX_ATOMS) return SR_ERR_UNSUPPORTED;
    if (lr->c != channels || out->c != channels || out->n != lr->n || index->n != lr->n || value->n != lr->n ||
        index->c != entries || value->c != entries || dict->n != 1 || dict->c != L || dict->h != k || dict->w != k ||
        (int64_t)lr->h * scale != out->h || (int64_t)lr->w * scale != out->w ||
        index->h != out->h || index->w != out->w || value->h != out->h || value->w != out->w) return SR_ERR_SHAPE;
    if (lr->n > 65535 || out->h > 4 * 65535 || out->w > (1 << 20)) return SR_ERR_UNSUPPORTED;
    if (lr->n == 0 || lr->h == 0 || lr->w == 0) return SR_OK;
    if (!lr->data || !index->data || !value->data || !dict->data || !out->data) return SR_ERR_NULL;
    if ((uintptr_t)lr->data % esize(lr->dtype) || (uintptr_t)out->data % esize(out->dtype) ||
        (uintptr_t)value->data % esize(value->dtype) || (uintptr_t)dict->data % 4) return SR_ERR_ALIGN;
    const size_t px = (size_t)out->h * out->w;
    const size_t out_b = (size_t)out->n * out->c * px * esize(out->dtype);
    if (overlap(out->data, out_b, lr->data, (size_t)lr->n * lr->c * lr->h * lr->w * esize(lr->dtype)) ||
        overlap(out->data, out_b, index->data, (size_t)index->n * entries * px) ||
        overlap(out->data, out_b, value->data, (size_t)value->n * entries * px * esize(value->dtype)) ||
        overlap(out->data, out_b, dict->data, (size_t)L * k * k * 4)) return SR_ERR_ALIAS;
    ListArgs a;
    a.lr = lr->data; a.index = (const unsigned char*)index->data; a.value = value->data;
    a.dict = (const float*)dict->data; a.out = out->data;
    a.N = lr->n; a.C = channels; a.h = lr->h; a.w = lr->w; a.H = out->h; a.W = out->w; a.s = scale; a.L = L; a.T = entries;
    const hipStream_t st = (hipStream_t)stream;
    hipError_t e;
    {
        AssembleArgs m;
        memset(&m, 0, sizeof(m));
        m.lr = lr->data; m.coeff = value->data; m.index = a.index; m.dict = a.dict; m.out = out->data;
        m.N = a.N; m.C = a.C; m.h = a.h; m.w = a.w; m.H = a.H; m.W = a.W; m.s = a.s; m.L = L; m.T = entries;
        m.n_fold = L; m.io_f16 = lr->dtype == SR_F16; m.coeff_dtype = SR_F16;
        for (int i = 0; i < L; ++i) { m.kept[i] = i; m.gamma[i] = 1.0f; }
        if (force_kernel != SR_KERNEL_GENERIC && mfma_list_supported(m, k, value->dtype == SR_F16)) {
            e = launch_mfma_list(m, st);
            return e == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
        }
        if (force_kernel == SR_KERNEL_MFMA) return SR_ERR_UNSUPPORTED;
    }
    if (value->dtype == SR_F16)
        e = lr->dtype == SR_F16 ? launch_list<__half, __half>(a, k, st) : launch_list<__half, float>(a, k, st);
    else
        e = lr->dtype == SR_F16 ? launch_list<float, __half>(a, k, st) : launch_list<float, float>(a, k, st);
    return e == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
}

extern "C" __attribute__((visibility("default")))
int sr_dict_assemble_list(const sr_tensor* lr, const sr_tensor* index, const sr_tensor* value, const sr_tensor* dict,
                          int L, int k, int scale, int channels, int entries, sr_tensor* out, void* stream) {
    return assemble_list(lr, index, value, dict, L, k, scale, channels, entries, out, stream, SR_KERNEL_AUTO);
}

extern "C" __attribute__((visibility("default")))
int sr_dict_assemble_list_ex(const sr_tensor* lr, const sr_tensor* index, const sr_tensor* value, const sr_tensor* dict,
                             int L, int k, int scale, int channels, int entries, sr_tensor* out, void* stream, int kernel) {
    if (kernel < SR_KERNEL_AUTO || kernel > SR_KERNEL_MFMA) return SR_ERR_UNSUPPORTED;
    return assemble_list(lr, index, value, dict, L, k, scale, channels, entries, out, stream, kernel);
}

// Offline dictionary selection (see include/sr_select.h): the normal equations of
// the LASSO regression of Eq. 7 on the GPU, and Alg. 1 on the host.
//
// GPU part.  A workgroup takes runs of 64 samples (lattice pixels).  For one run and
// one channel it first forms the responses r_{p,l} = Phi_{p,l} (D_l . B_p) of all
// atoms (one thread per sample and quarter of the atoms; the dictionary row is
// wave-uniform, so it comes through scalar loads) into an LDS tile [64][Lp], with
// the ground-truth pixel as one more column, then every thread accumulates its
// 4 x 4 blocks of the upper triangle of tile^T tile.  Sums are fp32 within a run and
// double across runs; each workgroup leaves its partial sums in the caller's
// scratch and a second kernel adds them in a fixed order.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <vector>

#include "../../include/sr_select.h"

namespace {

constexpr int NT = 256;          // threads per workgroup
constexpr int RUN = 64;          // samples per run
constexpr int NBMAX = 3;         // 4x4 blocks per thread: covers Lp = 132 (561 blocks)
constexpr int LPMAX = 132;       // SR_SELECT_MAX_ATOMS + 1, padded to a multiple of 4
constexpr int GRID = 512;        // workgroups (two per CU)

struct GramArgs {
    const float* up;
    const void* coeff;
    const float* dict;
    const float* target;
    double* ws;
    int N, C, H, W, L, stride, ny, nx;
    int Lp, nblk;                // padded column count (L + 1 -> multiple of 4), blocks in the upper triangle
};

int padded_columns(int L) { return 4 * ((L + 1 + 3) / 4); }
int upper_blocks(int Lp) { const int n = Lp / 4; return n * (n + 1) / 2; }

__device__ __forceinline__ float ldf(const float* p, size_t i) { return p[i]; }
__device__ __forceinline__ float ldf(const __half* p, size_t i) { return __half2float(p[i]); }
struct e4m3 { unsigned char bits; };        // 8-bit E4M3 storage, widened exactly by the conversion instruction
__device__ __forceinline__ float ldf(const e4m3* p, size_t i) { return __builtin_amdgcn_cvt_f32_fp8((int)p[i].bits, 0); }
__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// q-th 4x4 block of the upper triangle, row-major: (bi, bj) with bi <= bj
__device__ __forceinline__ void block_of(int q, int n4, int& bi, int& bj) {
    int r = 0, start = 0;
    while (start + (n4 - r) <= q) { start += n4 - r; ++r; }
    bi = r;
    bj = r + (q - start);
}

template <int K, typename TC>
__global__ __launch_bounds__(NT) void k_atom_gram(const GramArgs a) {
    constexpr int KK = K * K, R = (K - 1) / 2;
    __shared__ float tile[RUN * LPMAX];

    const int tid = threadIdx.x, si = tid & 63;
    const int g = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int Lp = a.Lp, n4 = Lp / 4;
    int bi[NBMAX], bj[NBMAX];
#pragma unroll
    for (int i = 0; i < NBMAX; ++i) {
        const int q = tid + NT * i;
        bi[i] = -1; bj[i] = 0;
        if (q < a.nblk) block_of(q, n4, bi[i], bj[i]);
    }
    double dacc[NBMAX][16];
#pragma unroll
    for (int i = 0; i < NBMAX; ++i)
#pragma unroll
        for (int e = 0; e < 16; ++e) dacc[i][e] = 0.0;

    const size_t plane = (size_t)a.H * a.W;
    const long long per_img = (long long)a.ny * a.nx, P = per_img * a.N;
    const long long nrun = (P + RUN - 1) / RUN;
    for (long long run = blockIdx.x; run < nrun; run += gridDim.x) {
        const long long s = run * RUN + si;
        const bool ok = s < P;
        int n = 0, Y = 0, X = 0;
        if (ok) {
            n = (int)(s / per_img);
            const int rem = (int)(s - (long long)n * per_img);
            const int iy = rem / a.nx;
            Y = iy * a.stride;
            X = (rem - iy * a.nx) * a.stride;
        }
        // the coefficients of this thread's atoms at its sample: the same for every channel
        float phi[LPMAX / 4];
#pragma unroll
        for (int i = 0; i < LPMAX / 4; ++i) {
            const int l = g + 4 * i;
            phi[i] = (ok && l < a.L)
                         ? ldf((const TC*)a.coeff, ((size_t)n * a.L + l) * plane + (size_t)Y * a.W + X) : 0.0f;
        }
        for (int c = 0; c < a.C; ++c) {
            // (1) responses of every atom at this thread's sample, plus the target column
            float patch[KK];
            const float* uplane = a.up + ((size_t)n * a.C + c) * plane;
#pragma unroll
            for (int dy = 0; dy < K; ++dy)
#pragma unroll
                for (int dx = 0; dx < K; ++dx) {
                    const int yy = clampi(Y + dy - R, 0, a.H - 1), xx = clampi(X + dx - R, 0, a.W - 1);
                    patch[dy * K + dx] = ok ? uplane[(size_t)yy * a.W + xx] : 0.0f;
                }
            const float hval = ok ? a.target[((size_t)n * a.C + c) * plane + (size_t)Y * a.W + X] : 0.0f;
#pragma unroll
            for (int i = 0; i < LPMAX / 4; ++i) {
                const int l = g + 4 * i;                // the same for the whole wavefront
                if (l < Lp) {
                    float r = 0.0f;
                    if (l < a.L) {
                        const float* d = a.dict + (size_t)l * KK;
                        float dot = 0.0f;
#pragma unroll
                        for (int j = 0; j < KK; ++j) dot = fmaf(d[j], patch[j], dot);
                        r = phi[i] * dot;
                    } else if (l == a.L) {
                        r = hval;
                    }
                    tile[si * Lp + l] = r;
                }
            }
            __syncthreads();
            // (2) this thread's blocks of tile^T tile over the 64 samples
            float acc[NBMAX][16];
#pragma unroll
            for (int i = 0; i < NBMAX; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc[i][e] = 0.0f;
            for (int ss = 0; ss < RUN; ++ss) {
#pragma unroll
                for (int i = 0; i < NBMAX; ++i)
                    if (bi[i] >= 0) {
                        const float4 u = *(const float4*)&tile[ss * Lp + 4 * bi[i]];
                        const float4 v = *(const float4*)&tile[ss * Lp + 4 * bj[i]];
                        const float uu[4] = {u.x, u.y, u.z, u.w}, vv[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
                        for (int e = 0; e < 4; ++e)
#pragma unroll
                            for (int f = 0; f < 4; ++f) acc[i][4 * e + f] = fmaf(uu[e], vv[f], acc[i][4 * e + f]);
                    }
            }
#pragma unroll
            for (int i = 0; i < NBMAX; ++i)
#pragma unroll
                for (int e = 0; e < 16; ++e) dacc[i][e] += (double)acc[i][e];
            __syncthreads();
        }
    }
#pragma unroll
    for (int i = 0; i < NBMAX; ++i)
        if (bi[i] >= 0) {
            double* dst = a.ws + ((size_t)blockIdx.x * a.nblk + (tid + NT * i)) * 16;
#pragma unroll
            for (int e = 0; e < 16; ++e) dst[e] = dacc[i][e];
        }
}

// Adds the workgroups' partial sums in workgroup order and scatters them into
// G (both triangles), b, hh; also stores the sample count.
__global__ __launch_bounds__(NT) void k_gram_reduce(const double* __restrict__ ws, int grid, int nblk, int n4, int L,
                                                    double M, double* __restrict__ normal) {
    const int idx = blockIdx.x * NT + threadIdx.x;
    if (idx == 0) normal[(size_t)L * L + L + 1] = M;
    if (idx >= nblk * 16) return;
    const int q = idx >> 4, e = idx & 15;
    int bi, bj;
    block_of(q, n4, bi, bj);
    double sum = 0.0;
    for (int w = 0; w < grid; ++w) sum += ws[((size_t)w * nblk + q) * 16 + e];
    const int row = 4 * bi + (e >> 2), col = 4 * bj + (e & 3);
    if (row > col) return;                      // diagonal blocks hold both triangles: keep the upper one
    if (col < L) {
        normal[(size_t)row * L + col] = sum;
        normal[(size_t)col * L + row] = sum;
    } else if (col == L) {
        if (row < L) normal[(size_t)L * L + row] = sum;
        else normal[(size_t)L * L + L] = sum;   // row == col == L: h^T h
    }
}

size_t tensor_elems(const sr_tensor* t) { return (size_t)t->n * t->c * t->h * t->w; }

// ---------------------------------------------------------------------------
// Host side of Alg. 1
// ---------------------------------------------------------------------------
typedef std::vector<double> vec;

// argmin (1/M)|h - R beta|^2 + lam |beta|_1 by cyclic coordinate descent on the
// normal equations (G: n x n row-major).  beta holds the start and the result.
void lasso_cd(const vec& G, const vec& b, int n, double M, double lam, vec& beta) {
    const double thr = 0.5 * lam * M, tol = 1e-13;
    for (int sweep = 0; sweep < 100000; ++sweep) {
        double dmax = 0.0, bmax = 0.0;
        for (int j = 0; j < n; ++j) {
            const double gjj = G[(size_t)j * n + j];
            double nw = 0.0;
            if (gjj > 0.0) {
                double dot = 0.0;
                for (int k = 0; k < n; ++k) dot += G[(size_t)j * n + k] * beta[k];
                const double rho = b[j] - (dot - gjj * beta[j]);
                nw = (rho > thr ? rho - thr : (rho < -thr ? rho + thr : 0.0)) / gjj;
            }
            dmax = fmax(dmax, fabs(nw - beta[j]));
            beta[j] = nw;
        }
        for (int j = 0; j < n; ++j) bmax = fmax(bmax, fabs(beta[j]));
        if (dmax <= tol * fmax(1.0, bmax)) break;
    }
}

int count_nonzero(const vec& v) {
    int c = 0;
    for (double x : v) c += x != 0.0;
    return c;
}

// Solves A x = y (n x n, row-major) by Gaussian elimination with partial pivoting;
// a vanishing pivot leaves that unknown at zero.
vec solve_dense(vec A, vec y, int n) {
    std::vector<int> piv_col;
    for (int col = 0; col < n; ++col) {
        int p = col;
        for (int r = col + 1; r < n; ++r)
            if (fabs(A[(size_t)r * n + col]) > fabs(A[(size_t)p * n + col])) p = r;
        if (fabs(A[(size_t)p * n + col]) < 1e-300) continue;
        if (p != col) {
            for (int k = 0; k < n; ++k) { const double t = A[(size_t)p * n + k]; A[(size_t)p * n + k] = A[(size_t)col * n + k]; A[(size_t)col * n + k] = t; }
            const double t = y[p]; y[p] = y[col]; y[col] = t;
        }
        for (int r = col + 1; r < n; ++r) {
            const double f = A[(size_t)r * n + col] / A[(size_t)col * n + col];
            if (f == 0.0) continue;
            for (int k = col; k < n; ++k) A[(size_t)r * n + k] -= f * A[(size_t)col * n + k];
            y[r] -= f * y[col];
        }
    }
    vec x(n, 0.0);
    for (int r = n - 1; r >= 0; --r) {
        double s = y[r];
        for (int k = r + 1; k < n; ++k) s -= A[(size_t)r * n + k] * x[k];
        const double d = A[(size_t)r * n + r];
        x[r] = fabs(d) < 1e-300 ? 0.0 : s / d;
    }
    return x;
}

}  // namespace

extern "C" __attribute__((visibility("default")))
size_t sr_atom_gram_workspace_bytes(int L) {
    if (L < 1 || L > SR_SELECT_MAX_ATOMS) return 0;
    return (size_t)GRID * upper_blocks(padded_columns(L)) * 16 * sizeof(double);
}

extern "C" __attribute__((visibility("default")))
int sr_atom_gram(const sr_tensor* up, const sr_tensor* coeff, const sr_tensor* dict, const sr_tensor* target,
                 int L, int k, int channels, int stride, void* workspace, size_t workspace_bytes,
                 double* normal, void* stream) {
    if (!up || !coeff || !dict || !target || !normal) return SR_ERR_NULL;
    if (up->dtype != SR_F32 || target->dtype != SR_F32 || dict->dtype != SR_F32 ||
        (coeff->dtype != SR_F32 && coeff->dtype != SR_F16 && coeff->dtype != SR_F8E4M3)) return SR_ERR_UNSUPPORTED;
    if ((k != 3 && k != 5 && k != 7) || L < 1 || L > SR_SELECT_MAX_ATOMS || channels < 1 ||
        channels > SR_MAX_CHANNELS || stride < 1) return SR_ERR_UNSUPPORTED;
    if (up->n < 0 || up->c < 0 || up->h < 0 || up->w < 0) return SR_ERR_SHAPE;
    if (up->c != channels || target->c != channels || coeff->c != L || dict->n != 1 || dict->c != L ||
        dict->h != k || dict->w != k || coeff->n != up->n || target->n != up->n ||
        coeff->h != up->h || coeff->w != up->w || target->h != up->h || target->w != up->w) return SR_ERR_SHAPE;
    if (up->h > (1 << 18) || up->w > (1 << 20) || up->n > 65535) return SR_ERR_UNSUPPORTED;
    const size_t need = sr_atom_gram_workspace_bytes(L);
    if (!workspace || workspace_bytes < need) return SR_ERR_SHAPE;
    if ((uintptr_t)workspace % 16 != 0 || (uintptr_t)normal % 8 != 0) return SR_ERR_ALIGN;
    const bool empty = tensor_elems(up) == 0;
    if (!empty) {
        if (!up->data || !coeff->data || !dict->data || !target->data) return SR_ERR_NULL;
        if ((uintptr_t)up->data % 4 || (uintptr_t)target->data % 4 || (uintptr_t)dict->data % 4 ||
            (uintptr_t)coeff->data % (coeff->dtype == SR_F16 ? 2 : (coeff->dtype == SR_F32 ? 4 : 1))) return SR_ERR_ALIGN;
    }
    GramArgs a;
    a.up = (const float*)up->data; a.coeff = coeff->data; a.dict = (const float*)dict->data;
    a.target = (const float*)target->data; a.ws = (double*)workspace;
    a.N = up->n; a.C = channels; a.H = up->h; a.W = up->w; a.L = L; a.stride = stride;
    a.ny = empty ? 0 : (up->h + stride - 1) / stride;
    a.nx = empty ? 0 : (up->w + stride - 1) / stride;
    a.Lp = padded_columns(L);
    a.nblk = upper_blocks(a.Lp);
    const hipStream_t st = (hipStream_t)stream;
#define SR_GRAM_LAUNCH(KS)                                                                                  \
    do {                                                                                                    \
        if (coeff->dtype == SR_F16) hipLaunchKernelGGL((k_atom_gram<KS, __half>), dim3(GRID), dim3(NT), 0, st, a);    \
        else if (coeff->dtype == SR_F32) hipLaunchKernelGGL((k_atom_gram<KS, float>), dim3(GRID), dim3(NT), 0, st, a); \
        else hipLaunchKernelGGL((k_atom_gram<KS, e4m3>), dim3(GRID), dim3(NT), 0, st, a);                             \
    } while (0)
    switch (k) {
    case 3:  SR_GRAM_LAUNCH(3); break;
    case 5:  SR_GRAM_LAUNCH(5); break;
    default: SR_GRAM_LAUNCH(7); break;
    }
#undef SR_GRAM_LAUNCH
    if (hipGetLastError() != hipSuccess) return SR_ERR_LAUNCH;
    const double M = (double)a.N * a.ny * a.nx * a.C;
    const int items = a.nblk * 16;
    hipLaunchKernelGGL(k_gram_reduce, dim3((items + NT - 1) / NT), dim3(NT), 0, st,
                       (const double*)workspace, GRID, a.nblk, a.Lp / 4, L, M, normal);
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
}

extern "C" __attribute__((visibility("default")))
int sr_select_atoms(const double* normal, int L, double alpha, double delta_alpha, double lambda0, double eps,
                    int* kept, int* n_kept, float* gamma, double* lambda_out) {
    if (!normal || !kept || !n_kept || !gamma) return SR_ERR_NULL;
    if (L < 1 || L > SR_SELECT_MAX_ATOMS || !(alpha > 0.0) || alpha > 1.0 || !(delta_alpha > 0.0) ||
        !(lambda0 > 0.0) || !(eps >= 0.0)) return SR_ERR_UNSUPPORTED;
    vec G(normal, normal + (size_t)L * L), b(normal + (size_t)L * L, normal + (size_t)L * L + L);
    const double M = normal[(size_t)L * L + L + 1];
    if (!(M > 0.0)) return SR_ERR_UNSUPPORTED;
    std::vector<int> active(L);
    for (int i = 0; i < L; ++i) active[i] = i;
    vec gamma_tot(L, 1.0);
    double alpha_t = 1.0, lam = lambda0;
    while (alpha_t > alpha + 1e-12 && !active.empty()) {
        alpha_t = fmax(alpha, alpha_t - delta_alpha);
        const double want = alpha_t * L;
        const int n = (int)active.size();
        vec Ga((size_t)n * n), ba(n);
        for (int i = 0; i < n; ++i) {
            ba[i] = b[active[i]];
            for (int j = 0; j < n; ++j) Ga[(size_t)i * n + j] = G[(size_t)active[i] * L + active[j]];
        }
        auto solve = [&](double lm, vec& bt) {
            bt.assign(n, 1.0);
            lasso_cd(Ga, ba, n, M, lm, bt);
            return count_nonzero(bt);
        };
        // lambda doubles until few enough atoms survive
        double lam_lo = 0.5 * lam, lam_hi = lam;
        vec beta;
        int cnt = solve(lam_hi, beta);
        while (cnt > want) {
            lam_lo = lam_hi;
            lam_hi *= 2.0;
            cnt = solve(lam_hi, beta);
        }
        // bisection towards the target count, keeping a solution that meets it
        for (int it = 0; it < 60 && fabs(want - cnt) > eps * L && want - cnt >= 1.0; ++it) {
            const double mid = 0.5 * (lam_lo + lam_hi);
            vec bm;
            const int cm = solve(mid, bm);
            if (cm > want) lam_lo = mid;
            else { lam_hi = mid; beta = bm; cnt = cm; }
        }
        lam = lam_hi;
        std::vector<int> keep;
        for (int i = 0; i < n; ++i)
            if (beta[i] != 0.0) keep.push_back(i);
        if (keep.empty()) { active.clear(); break; }
        // regression scales of the kept atoms (Eq. 9): G_SS gamma = b_S
        const int m = (int)keep.size();
        vec Gs((size_t)m * m), bs(m);
        for (int i = 0; i < m; ++i) {
            bs[i] = ba[keep[i]];
            for (int j = 0; j < m; ++j) Gs[(size_t)i * m + j] = Ga[(size_t)keep[i] * n + keep[j]];
        }
        const vec gam = solve_dense(Gs, bs, m);
        std::vector<int> S(m);
        for (int i = 0; i < m; ++i) { S[i] = active[keep[i]]; gamma_tot[S[i]] *= gam[i]; }
        // the kept atoms' coefficients are rescaled by gamma from here on
        for (int i = 0; i < m; ++i) {
            b[S[i]] *= gam[i];
            for (int j = 0; j < m; ++j) G[(size_t)S[i] * L + S[j]] *= gam[i] * gam[j];
        }
        active = S;
    }
    *n_kept = (int)active.size();
    for (size_t i = 0; i < active.size(); ++i) { kept[i] = active[i]; gamma[i] = (float)gamma_tot[active[i]]; }
    if (lambda_out) *lambda_out = lam;
    return SR_OK;
}

// Offline dictionary selection (see include/sr_select.h): the normal equations of
// the LASSO regression of Eq. 7 on the GPU, and Alg. 1 on the host.
//
// GPU part.  A workgroup takes runs of 64 samples (lattice pixels).  For one run and
// one channel it first forms the responses r_{p,l} = Phi_{p,l} (D_l . B_p) of all
// atoms into an LDS tile [column][sample], with the ground-truth pixel as one more
// column.  tile^T tile is a dense contraction over the samples and runs on the
// matrix cores: the upper triangle is cut into 16 x 16 blocks, dealt to four
// wavefronts, and each block takes 16 v_mfma_f32_16x16x4_f32 steps per run (a lane
// reads four consecutive samples of its column with one 16-byte LDS load and spends
// them on four steps; which sample goes to which step does not matter to the sum as
// long as both operands agree).  Sums are fp32 within a run and double across runs;
// each workgroup leaves its partial sums in the caller's scratch and a second kernel
// adds them in a fixed order.
//
// Two forms of the first kernel.  k_atom_gram_rows (lattice strides up to 4): runs
// are segments of one lattice row, eight wavefronts per workgroup split into four
// that form responses (their dot products on the matrix cores too) and four that
// contract, all global loads coalesced and parked in LDS.  k_atom_gram (any stride):
// runs are 64 consecutive samples in lattice order, one thread per sample gathers
// its neighbourhood, the dictionary row comes through scalar loads, and the same
// four wavefronts form the responses and contract them.
#include <hip/hip_fp16.h>
#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include <algorithm>
#include <mutex>
#include <vector>

#include "../../include/sr_select.h"

namespace {

constexpr int NT = 256;          // threads per workgroup
constexpr int RUN = 64;          // samples per run
constexpr int TSS = RUN + 4;     // floats per tile column: 16-byte loads of 16 columns x 4 sample groups miss each other's banks
constexpr int GRID = 512;        // workgroups (two per CU)

typedef float f32x4 __attribute__((ext_vector_type(4)));

struct GramArgs {
    const float* up;
    const void* coeff;
    const float* dict;
    const float* target;
    double* ws;
    int N, C, H, W, L, stride, ny, nx;
    int n16, ntile;              // 16-column blocks covering L + 1 columns, blocks in the upper triangle
};

int column_blocks(int L) { return (L + 1 + 15) / 16; }
int upper_blocks(int n) { return n * (n + 1) / 2; }

struct e4m3 { unsigned char bits; };        // 8-bit E4M3 storage, widened exactly by the conversion instruction
__device__ __forceinline__ float widen(float v) { return v; }
__device__ __forceinline__ float widen(__half v) { return __half2float(v); }
__device__ __forceinline__ float widen(e4m3 v) { return __builtin_amdgcn_cvt_f32_fp8((int)v.bits, 0); }
struct bf16v { unsigned short bits; };      // bfloat16 storage: the upper half of a binary32
__device__ __forceinline__ float widen(bf16v v) { return __uint_as_float((unsigned)v.bits << 16); }
__device__ __forceinline__ int clampi(int v, int lo, int hi) { return v < lo ? lo : (v > hi ? hi : v); }

// q-th block of the upper triangle of an n x n block matrix, row-major: (bi, bj) with bi <= bj
__device__ __forceinline__ void block_of(int q, int n, int& bi, int& bj) {
    int r = 0, start = 0;
    while (start + (n - r) <= q) { start += n - r; ++r; }
    bi = r;
    bj = r + (q - start);
}

// N16: 16-column blocks the LDS tile has room for (2, 5 or 9; the frame's own count
// a.n16 may be smaller: the columns beyond it are computed as zeros and never read).
// Up to 5 blocks there are two LDS tiles, so that one barrier per run and channel is
// enough.  The response loop has no branches: atoms past L read the last dictionary
// row with a zero coefficient, so the scalar loads of one atom's row overlap the
// multiply-adds of the one before.
template <int K, typename TC, int N16>
__global__ __launch_bounds__(NT, (N16 <= 5 && K <= 5) ? 2 : 1) void k_atom_gram(const GramArgs a) {
    constexpr int KK = K * K, R = (K - 1) / 2;
    constexpr int NTW = N16 == 2 ? 1 : (N16 == 5 ? 4 : 12);     // blocks per wavefront
    constexpr int NBUF = N16 <= 5 ? 2 : 1;
    constexpr int NPHI = N16 * 4;                     // columns per thread (one wavefront takes every fourth)
    __shared__ float tile[NBUF][N16 * 16 * TSS];

    const int tid = threadIdx.x, si = tid & 63, c16 = tid & 15, kq = (tid >> 4) & 3;
    const int g = __builtin_amdgcn_readfirstlane(tid >> 6);
    // blocks g, g + 4, ... of the upper triangle; a wavefront with fewer blocks than
    // the others repeats the last block (and does not store it) so that the
    // matrix-core loop has no branches
    int bi[NTW], bj[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        const int q = g + 4 * t;
        block_of(q < a.ntile ? q : a.ntile - 1, a.n16, bi[t], bj[t]);
    }
    double dacc[NTW][4];
#pragma unroll
    for (int t = 0; t < NTW; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) dacc[t][e] = 0.0;

    const size_t plane = (size_t)a.H * a.W;
    const long long per_img = (long long)a.ny * a.nx, P = per_img * a.N;
    const long long nrun = (P + RUN - 1) / RUN;

    // A thread's sample: validity, image, and the offsets of its clamped k x k
    // neighbourhood (nearest pixel outside the image) within a plane.
    // (a sample past the end is clamped to the last one, so that every load has a
    // valid address and needs no branch; its responses are zeroed instead)
    struct Sample { bool ok; int n; size_t row[K], col[K], centre; };
    auto sample_of = [&](long long run) {
        const long long s = run * RUN + si;
        Sample p;
        p.ok = s < P;
        const long long sc = p.ok ? s : P - 1;
        p.n = (int)(sc / per_img);
        const int rem = (int)(sc - (long long)p.n * per_img);
        const int iy = rem / a.nx;
        const int Y = iy * a.stride, X = (rem - iy * a.nx) * a.stride;
#pragma unroll
        for (int d = 0; d < K; ++d) {
            p.row[d] = (size_t)clampi(Y + d - R, 0, a.H - 1) * a.W;
            p.col[d] = clampi(X + d - R, 0, a.W - 1);
        }
        p.centre = (size_t)Y * a.W + X;
        return p;
    };
    // The coefficients of this thread's atoms at its sample (the same for every
    // channel), the k x k neighbourhood and the target pixel: requested here as
    // stored, widened and masked only where they are used, so that a request never
    // waits for its own data.
    auto load_phi = [&](const Sample& p, TC (&raw)[NPHI]) {
        const TC* base = (const TC*)a.coeff + (size_t)p.n * a.L * plane + p.centre;
#pragma unroll
        for (int i = 0; i < NPHI; ++i) {
            const int l = g + 4 * i;
            raw[i] = base[(size_t)(l < a.L ? l : a.L - 1) * plane];
        }
    };
    auto finish_phi = [&](const Sample& p, const TC (&raw)[NPHI], float (&phi)[NPHI]) {
#pragma unroll
        for (int i = 0; i < NPHI; ++i) phi[i] = (p.ok && g + 4 * i < a.L) ? widen(raw[i]) : 0.0f;
    };
    auto load_patch = [&](const Sample& p, int c, float (&patch)[KK], float& h) {
        const size_t pl = ((size_t)p.n * a.C + c) * plane;
        const float* uplane = a.up + pl;
#pragma unroll
        for (int dy = 0; dy < K; ++dy)
#pragma unroll
            for (int dx = 0; dx < K; ++dx) patch[dy * K + dx] = uplane[p.row[dy] + p.col[dx]];
        h = a.target[pl + p.centre];
    };

    long long run = blockIdx.x;
    if (run < nrun) {
        // One iteration per (run, channel).  The operands of the next iteration are
        // requested before the matrix-core phase of this one and used after it.
        Sample smp = sample_of(run), smp_n = smp;
        TC raw_n[NPHI];
        float phi[NPHI], patch[KK], patch_n[KK], hval, hval_n;
        load_phi(smp, raw_n);
        load_patch(smp, 0, patch, hval);
        finish_phi(smp, raw_n, phi);
        hval = smp.ok ? hval : 0.0f;
        hval_n = 0.0f;
#pragma unroll
        for (int j = 0; j < KK; ++j) patch_n[j] = 0.0f;
        int c = 0, buf = 0;
        for (;;) {
            // (1) responses of every atom at this thread's sample, plus the target column
            float* T = tile[buf];
            // (the dictionary row of the next atom is requested before the multiply-adds
            // of this one: scalar loads return out of order, so a wait is always for all
            // of them, and the scheduling fences keep the request one atom ahead)
            float drow[KK], drow_n[KK];
            auto dict_row = [&](int i, float (&d)[KK]) {
                const int l = g + 4 * i;                // the same for the whole wavefront
                const float* src = a.dict + (size_t)(l < a.L ? l : a.L - 1) * KK;
#pragma unroll
                for (int j = 0; j < KK; ++j) d[j] = src[j];
            };
            dict_row(0, drow);
#pragma unroll
            for (int i = 0; i < NPHI; ++i) {
                const int l = g + 4 * i;
                if (i + 1 < NPHI) dict_row(i + 1, drow_n);
                __builtin_amdgcn_sched_barrier(0);
                float dot = 0.0f;
#pragma unroll
                for (int j = 0; j < KK; ++j) dot = fmaf(drow[j], patch[j], dot);
                T[l * TSS + si] = l == a.L ? hval : phi[i] * dot;      // phi is zero past L
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int j = 0; j < KK; ++j) drow[j] = drow_n[j];
            }
            __syncthreads();
            int c_n = c + 1;
            long long run_n = run;
            if (c_n == a.C) { c_n = 0; run_n = run + gridDim.x; }
            const bool more = run_n < nrun;
            if (more) {
                if (c_n == 0) {
                    smp_n = sample_of(run_n);
                    load_phi(smp_n, raw_n);
                }
                load_patch(smp_n, c_n, patch_n, hval_n);
            }
            // (2) this wavefront's blocks of tile^T tile over the 64 samples
            f32x4 acc[NTW];
#pragma unroll
            for (int t = 0; t < NTW; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
            // (blocks go four at a time: their operands are read together and their
            // steps interleaved, so that a step never waits for the one before it)
            constexpr int TG = NTW < 4 ? NTW : 4;
#pragma unroll
            for (int sg = 0; sg < RUN / 16; ++sg) {
#pragma unroll
                for (int t0 = 0; t0 < NTW; t0 += TG) {
                    float4 u[TG], v[TG];
#pragma unroll
                    for (int t = 0; t < TG; ++t) {
                        u[t] = *(const float4*)&T[(16 * bi[t0 + t] + c16) * TSS + 16 * sg + 4 * kq];
                        v[t] = *(const float4*)&T[(16 * bj[t0 + t] + c16) * TSS + 16 * sg + 4 * kq];
                    }
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].x, v[t].x, acc[t0 + t], 0, 0, 0);
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].y, v[t].y, acc[t0 + t], 0, 0, 0);
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].z, v[t].z, acc[t0 + t], 0, 0, 0);
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].w, v[t].w, acc[t0 + t], 0, 0, 0);
                }
            }
#pragma unroll
            for (int t = 0; t < NTW; ++t)
#pragma unroll
                for (int e = 0; e < 4; ++e) dacc[t][e] += (double)acc[t][e];
            if (NBUF == 1) __syncthreads();
            else buf ^= 1;
            if (!more) break;
            if (c_n == 0) {
                smp = smp_n;
                finish_phi(smp, raw_n, phi);
            }
#pragma unroll
            for (int j = 0; j < KK; ++j) patch[j] = patch_n[j];
            hval = smp.ok ? hval_n : 0.0f;
            c = c_n;
            run = run_n;
        }
    }
    // lane (c16, kq), register e of block (bi, bj) holds row 16 bi + 4 kq + e, column 16 bj + c16
#pragma unroll
    for (int t = 0; t < NTW; ++t)
        if (g + 4 * t < a.ntile) {
            double* dst = a.ws + ((size_t)blockIdx.x * a.ntile + (g + 4 * t)) * 256 + si * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[e] = dacc[t][e];
        }
}

// ---------------------------------------------------------------------------
// Second form of the kernel, for lattice strides up to 4 (every pixel down to every
// fourth): workgroups of eight wavefronts, one or two per CU.  Four wavefronts form the
// responses of one (run, channel) while the other four contract the tile of the
// one before; two LDS tiles, one barrier per iteration.  A run is 64 consecutive
// lattice samples of ONE lattice row, so the k image rows it needs are contiguous
// segments and every atom's 64 coefficients one or a few cache lines.
//
// Every global load is coalesced, requested a whole iteration before its data is
// parked in LDS and two before it is read, and the duty is split by role so that
// neither kind of wavefront waits for the other: the response wavefronts stage the
// row segments of the next channel, the contracting ones fetch the coefficients and
// target pixels of the next run (one atom's 64 samples per load) and park them
// widened and masked.  The dot products D_l . B_p of the responses are a contraction
// too, (samples x taps) . (taps x atoms), and run on the matrix cores with the
// dictionary as a register-resident operand: no per-atom scalar loads or broadcasts,
// whose latency a single wavefront per SIMD cannot hide.
// ---------------------------------------------------------------------------
constexpr int NT2 = 512;         // four response + four contraction wavefronts
constexpr int GRID2 = 256;       // one workgroup per CU (two where registers and LDS allow)
constexpr int STMAX = 4;         // largest lattice stride whose row segments are staged

// floats of dynamic LDS: tile[2], coefficients of a run [1 or 2], its targets [2], staged segments [2]
constexpr size_t rows_lds_floats(int k, int n16, int channels) {
    return (size_t)(2 + (channels == 1 ? 2 : 1)) * n16 * 16 * TSS + 2 * (size_t)channels * RUN +
           2 * (((size_t)k * (63 * STMAX + k) + 3) & ~(size_t)3);
}

// Five column blocks (64 to 79 atoms, the paper's 72 among them): the 15 blocks of
// the upper triangle dealt to the four contracting wavefronts so that a wavefront's
// blocks share their operands.  Wavefront w reads the column blocks col[w][0 .. nc)
// of the tile (one 16-byte LDS load each per 16 samples: 14 loads for the 15 blocks,
// where separate operands for every block would take 30) and block t multiplies
// operand u[w][t] by operand v[w][t]; q is the block's row-major number in the
// upper triangle.
struct Deal5 { int nc, nb, col[4], u[4], v[4], q[4]; };
constexpr Deal5 deal5(int w) {
    return w == 0 ? Deal5{3, 4, {0, 1, 2, 0}, {0, 0, 1, 0}, {0, 1, 1, 2}, {0, 1, 5, 2}}        // 00 01 11 02
         : w == 1 ? Deal5{3, 4, {1, 2, 3, 0}, {1, 1, 2, 0}, {1, 2, 2, 1}, {9, 10, 12, 6}}      // 22 23 33 12
         : w == 2 ? Deal5{4, 4, {1, 2, 3, 4}, {3, 2, 1, 0}, {3, 3, 3, 3}, {14, 13, 11, 8}}     // 44 34 24 14
                  : Deal5{4, 3, {0, 1, 3, 4}, {0, 0, 1, 0}, {2, 3, 2, 0}, {3, 4, 7, 0}};       // 03 04 13
}
template <int W>
__device__ __forceinline__ void contract5(const float* T, int c16, int kq, f32x4 (&acc)[4]) {
    constexpr Deal5 d = deal5(W);
#pragma unroll
    for (int sg = 0; sg < RUN / 16; ++sg) {
        float4 x[4];
#pragma unroll
        for (int i = 0; i < d.nc; ++i) x[i] = *(const float4*)&T[(16 * d.col[i] + c16) * TSS + 16 * sg + 4 * kq];
#pragma unroll
        for (int t = 0; t < d.nb; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[d.u[t]].x, x[d.v[t]].x, acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < d.nb; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[d.u[t]].y, x[d.v[t]].y, acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < d.nb; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[d.u[t]].z, x[d.v[t]].z, acc[t], 0, 0, 0);
#pragma unroll
        for (int t = 0; t < d.nb; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(x[d.u[t]].w, x[d.v[t]].w, acc[t], 0, 0, 0);
    }
}
// block number of slot t of wavefront w in that deal, -1: none
__device__ __forceinline__ int deal5_block(int w, int t) {
    const Deal5 d = w == 0 ? deal5(0) : (w == 1 ? deal5(1) : (w == 2 ? deal5(2) : deal5(3)));
    return t < d.nb ? d.q[t] : -1;
}

template <int K, typename TC, int N16>
__global__ __launch_bounds__(NT2, (N16 <= 5 && K <= 5) ? 4 : 2) void k_atom_gram_rows(const GramArgs a) {
    constexpr int KK = K * K, R = (K - 1) / 2;
    constexpr int NTW = N16 == 2 ? 1 : (N16 == 5 ? 4 : 12);     // blocks per contracting wavefront
    constexpr int NPW = N16 * 4;                      // atoms whose coefficients one contracting wavefront fetches
    constexpr int TILE = N16 * 16 * TSS;
    constexpr int PSZ = (K * (63 * STMAX + K) + 3) & ~3;   // staged row segments of one run and channel (whole 16 bytes)
    constexpr int MM = (PSZ + 255) / 256;             // staged elements per thread
    // Coefficients of a run, widened and masked, laid out like a tile.  With one channel a
    // run lasts one iteration and the copy for the next run is written while this one is
    // read: two copies.  Otherwise the last channel's iteration writes, the first reads.
    const int phbuf = a.C == 1 ? 2 : 1;
    extern __shared__ float lds[];                    // tile[2][TILE], phi[phbuf][TILE], target[2][C][RUN], stage[2][PSZ]
    float* const PH = lds + 2 * TILE;
    // The run's target pixels, every channel.  They are read in every iteration of the run,
    // the last of which overlaps the parking of the next run's: always two copies.
    float* const TGT = PH + phbuf * TILE;
    float* const stage = TGT + 2 * a.C * RUN;

    const int tid = threadIdx.x, si = tid & 63, c16 = tid & 15, kq = (tid >> 4) & 3;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), g = wave & 3;
    const bool contracts = wave >= 4;

    const size_t plane = (size_t)a.H * a.W;
    const int WD = 63 * a.stride + K;                 // columns of a staged segment
    const int nseg = (a.nx + RUN - 1) / RUN;          // runs per lattice row
    const long long rpi = (long long)a.ny * nseg, nrun = rpi * a.N;
    // iterations of this workgroup: its runs blockIdx.x, blockIdx.x + gridDim.x, ... times the channels
    const long long my_runs = (long long)blockIdx.x < nrun ? (nrun - blockIdx.x + gridDim.x - 1) / gridDim.x : 0;
    const long long n_it = my_runs * a.C;
    if (n_it == 0) {
        // nothing to add: the partial sums must still be defined
        if (contracts) {
#pragma unroll
            for (int t = 0; t < NTW; ++t)
                if (g + 4 * t < a.ntile) {
                    double* dst = a.ws + ((size_t)blockIdx.x * a.ntile + (g + 4 * t)) * 256 + si * 4;
#pragma unroll
                    for (int e = 0; e < 4; ++e) dst[e] = 0.0;
                }
        }
        return;
    }

    // A run: image, lattice row, 64-sample segment of that row.  This workgroup's
    // runs are gridDim.x apart; the step is pre-split so that no division is left in the
    // loop.  All of it is scalar.
    struct Run { int n, iy, seg; };
    const int G = gridDim.x;
    const int step_n = (int)(G / rpi), step_r = (int)(G - step_n * rpi);
    const int step_y = step_r / nseg, step_s = step_r - step_y * nseg;
    auto advance = [&](Run r) {
        r.seg += step_s;
        if (r.seg >= nseg) { r.seg -= nseg; r.iy += 1; }
        r.iy += step_y;
        if (r.iy >= a.ny) { r.iy -= a.ny; r.n += 1; }
        r.n += step_n;
        return r;
    };
    const int t2 = tid & 255;                            // 0 .. 255 among the wavefronts of one kind
    // staged elements of this thread: e = t2 + 256 m  <->  (row dy, column q) of the segment
    int sdy[MM], sq[MM];
#pragma unroll
    for (int m = 0; m < MM; ++m) {
        const int e = t2 + 256 * m;
        sdy[m] = e / WD;
        sq[m] = e - sdy[m] * WD;
        if (sdy[m] >= K) sdy[m] = K - 1;                 // past K * WD: a valid address, not stored
    }
    Run run0;
    {
        run0.n = (int)(blockIdx.x / rpi);
        const int rr = (int)(blockIdx.x - (long long)run0.n * rpi);
        run0.iy = rr / nseg;
        run0.seg = rr - run0.iy * nseg;
    }
    // this lane's sample of a run: pixel index within a plane (fewer than 2^30 pixels, checked
    // on the host), and whether it exists (past the end of the row: clamped to the last one,
    // zeroed where it is parked)
    auto sample_of = [&](const Run& r, bool& ok) {
        const int X = (r.seg * RUN + si) * a.stride, Xl = (a.nx - 1) * a.stride;
        ok = X <= Xl;
        return (unsigned)(r.iy * a.stride) * (unsigned)a.W + (unsigned)(ok ? X : Xl);
    };

    if (!contracts) {
        // Response wavefront g takes samples 16 g .. 16 g + 15 of the run and all atoms.
        // A operand: read from the staged segment; B operand: the dictionary, in
        // registers for the whole kernel.  A lane ends up with four consecutive samples
        // of one atom per 16-atom block, which it scales by the coefficients and writes
        // to the tile with one 16-byte store.
        constexpr int KS = (KK + 3) / 4;               // 4-tap steps of v_mfma_f32_16x16x4_f32
        const int kq4 = 16 * g + 4 * kq;               // first of this lane's four samples
        // lane (c16, kq) holds tap 4 ks + kq of atom 16 nb + c16
        float Bd[N16][KS];
#pragma unroll
        for (int nb = 0; nb < N16; ++nb)
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const int l = 16 * nb + c16, tap = 4 * ks + kq;
                Bd[nb][ks] = (l < a.L && tap < KK) ? a.dict[(size_t)l * KK + tap] : 0.0f;
            }
        // offset of this lane's A operand within a staged segment: sample 16 g + c16, tap 4 ks + kq
        int aoff[KS];
        bool atap[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int tap = 4 * ks + kq;
            atap[ks] = tap < KK;
            const int tc = atap[ks] ? tap : 0, dy = tc / K, dx = tc - dy * K;
            aoff[ks] = dy * WD + (16 * g + c16) * a.stride + dx;
        }
        const int tcol = a.L >> 4;                       // the block that holds column L (the target) ...
        const bool holds_target = c16 == (a.L & 15);    // ... and the lanes that hold it there
        // Staging: the segment's elements e = t2 + 256 m of this thread, requested a whole
        // iteration before they are parked, which is an iteration before they are read.
        struct Fetch { float sv[MM]; };
        auto fetch = [&](const Run& r, int c, Fetch& f) {
            const int Y = r.iy * a.stride, X0 = r.seg * RUN * a.stride;
            const char* pl = (const char*)(a.up + ((size_t)r.n * a.C + c) * plane);      // wave-uniform
#pragma unroll
            for (int m = 0; m < MM; ++m) {
                const unsigned o = (unsigned)clampi(Y + sdy[m] - R, 0, a.H - 1) * (unsigned)a.W +
                                   (unsigned)clampi(X0 - R + sq[m], 0, a.W - 1);
                f.sv[m] = *(const float*)(pl + 4u * o);
            }
        };
        auto park = [&](const Fetch& f, float* S) {
#pragma unroll
            for (int m = 0; m < MM; ++m)
                if (t2 + 256 * m < K * WD) S[t2 + 256 * m] = f.sv[m];
        };
        Run ra = run0;
        int ca = 0;
        long long ia = 0;
        auto step_ahead = [&]() {
            ++ia;
            if (++ca == a.C) { ca = 0; ra = advance(ra); }
        };
        Fetch f;
        fetch(ra, ca, f);
        park(f, stage);
        step_ahead();
        bool parked = ia >= n_it;
        if (!parked) fetch(ra, ca, f);
        step_ahead();
        float phi[N16][4];
        int c = 0, pp = 0, tp = 0;
        const float* H = TGT;                            // targets of the current run
        __syncthreads();                                // iteration 0 is staged, the first coefficients parked
        for (long long it = 0; it < n_it; ++it) {
            const int buf = (int)(it & 1);
            const float* P = stage + buf * PSZ;
            if (!parked) park(f, stage + (buf ^ 1) * PSZ);  // iteration it + 1
            parked = ia >= n_it;                            // ia == it + 2
            if (!parked) fetch(ra, ca, f);
            step_ahead();
            if (c == 0) {                                // a new run: its coefficients
                const float* Q = PH + pp * TILE;
                H = TGT + tp * a.C * RUN;
                tp ^= 1;
#pragma unroll
                for (int nb = 0; nb < N16; ++nb) {
                    const float4 q = *(const float4*)&Q[(16 * nb + c16) * TSS + kq4];
                    phi[nb][0] = q.x; phi[nb][1] = q.y; phi[nb][2] = q.z; phi[nb][3] = q.w;
                }
                pp ^= phbuf - 1;
            }
            float av[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) av[ks] = P[aoff[ks]];
            const float4 h = *(const float4*)&H[c * RUN + kq4];
            f32x4 dot[N16];
#pragma unroll
            for (int nb = 0; nb < N16; ++nb) dot[nb] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
                const float av_k = atap[ks] ? av[ks] : 0.0f;
#pragma unroll
                for (int nb = 0; nb < N16; ++nb)
                    dot[nb] = __builtin_amdgcn_mfma_f32_16x16x4f32(av_k, Bd[nb][ks], dot[nb], 0, 0, 0);
            }
            // responses (and the target column) into the tile: column 16 nb + c16, samples kq4 .. kq4 + 3
            float* T = lds + buf * TILE;
#pragma unroll
            for (int nb = 0; nb < N16; ++nb) {
                float4 o;
                o.x = phi[nb][0] * dot[nb][0];          // phi is zero past L and past the end of the row
                o.y = phi[nb][1] * dot[nb][1];
                o.z = phi[nb][2] * dot[nb][2];
                o.w = phi[nb][3] * dot[nb][3];
                if (nb == tcol && holds_target) o = h;
                *(float4*)&T[(16 * nb + c16) * TSS + kq4] = o;
            }
            __syncthreads();                            // this tile is complete
            c = c + 1 == a.C ? 0 : c + 1;
        }
        return;
    }

    // ---- contracting wavefronts ----
    // Coefficients of a run: this lane's sample, atoms g, g + 4, ...; requested a whole
    // iteration before they are parked
    // ... and its target pixels of channels g, g + 4, ...
    constexpr int NCW = (SR_MAX_CHANNELS + 3) / 4;
    struct Fetch { TC raw[NPW]; float h[NCW]; bool ok; int pp, tp; };
    auto fetch = [&](const Run& r, Fetch& f) {
        const unsigned centre = sample_of(r, f.ok);
#pragma unroll
        for (int j = 0; j < NCW; ++j) {
            const int c = g + 4 * j;
            f.h[j] = a.target[((size_t)r.n * a.C + (c < a.C ? c : a.C - 1)) * plane + centre];
        }
        const TC* img = (const TC*)a.coeff + (size_t)r.n * a.L * plane;
#pragma unroll
        for (int j = 0; j < NPW; ++j) {
            const int l = g + 4 * j;
            f.raw[j] = img[(size_t)(l < a.L ? l : a.L - 1) * plane + centre];            // plane: wave-uniform
        }
    };
    auto park = [&](const Fetch& f) {
        float* Q = PH + f.pp * TILE;
        float* Hn = TGT + f.tp * a.C * RUN;
#pragma unroll
        for (int j = 0; j < NCW; ++j)
            if (g + 4 * j < a.C) Hn[(g + 4 * j) * RUN + si] = f.ok ? f.h[j] : 0.0f;
#pragma unroll
        for (int j = 0; j < NPW; ++j) {
            const int l = g + 4 * j;
            Q[l * TSS + si] = (f.ok && l < a.L) ? widen(f.raw[j]) : 0.0f;
        }
    };

    // Blocks g, g + 4, ... of the upper triangle; a wavefront with fewer blocks than the
    // others repeats the last block (and does not store it) so that the matrix-core loop
    // has no branches.
    int bi[NTW], bj[NTW];
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        const int q = g + 4 * t;
        block_of(q < a.ntile ? q : a.ntile - 1, a.n16, bi[t], bj[t]);
    }
    double dacc[NTW][4];
#pragma unroll
    for (int t = 0; t < NTW; ++t)
#pragma unroll
        for (int e = 0; e < 4; ++e) dacc[t][e] = 0.0;
    const bool shared_operands = N16 == 5 && a.n16 == 5;     // the deal of deal5() instead

    // The run whose coefficients are requested next, the first iteration that reads them
    // and the copy they go to.  Requested in iteration ia - 3, parked in iteration ia - 2
    // (after the barrier that ends the last read of a single copy, see phbuf).
    Run ra = run0;
    long long ia = 0;
    int ppa = 0, tpa = 0;
    auto step_ahead = [&]() {
        ia += a.C;
        ra = advance(ra);
        ppa ^= phbuf - 1;
        tpa ^= 1;
    };
    Fetch f;
    fetch(ra, f);
    f.pp = ppa; f.tp = tpa;
    park(f);
    step_ahead();
    bool parked = true;                                 // nothing waits in f
    if (ia < n_it && ia <= 2) {                         // a run that starts in iteration 1 or 2: request now
        fetch(ra, f);
        f.pp = ppa; f.tp = tpa;
        parked = false;
        const bool now = ia == 1;                       // ... iteration 1: park before iteration 0 ends
        step_ahead();
        __syncthreads();                                // iteration 0 is staged
        if (now) {
            park(f);
            parked = true;
            if (ia < n_it && ia <= 2) { fetch(ra, f); f.pp = ppa; f.tp = tpa; parked = false; step_ahead(); }
        }
    } else {
        __syncthreads();                                // iteration 0 is staged
    }
    for (long long it = 0; it < n_it; ++it) {
        __syncthreads();                                // the tile of iteration it is complete, it + 1 is staged
        const int buf = (int)(it & 1);
        if (!parked) { park(f); parked = true; }        // read from iteration it + 2 on
        if (ia < n_it && ia <= it + 3) { fetch(ra, f); f.pp = ppa; f.tp = tpa; parked = false; step_ahead(); }
        const float* T = lds + buf * TILE;
        f32x4 acc[NTW];
#pragma unroll
        for (int t = 0; t < NTW; ++t) acc[t] = f32x4{0.0f, 0.0f, 0.0f, 0.0f};
        constexpr int TG = NTW < 4 ? NTW : 4;           // blocks go four at a time, their steps interleaved
        if constexpr (N16 == 5) {
            if (shared_operands) {
                switch (g) {
                case 0:  contract5<0>(T, c16, kq, acc); break;
                case 1:  contract5<1>(T, c16, kq, acc); break;
                case 2:  contract5<2>(T, c16, kq, acc); break;
                default: contract5<3>(T, c16, kq, acc); break;
                }
            }
        }
        if (!shared_operands) {
#pragma unroll
            for (int sg = 0; sg < RUN / 16; ++sg) {
#pragma unroll
                for (int t0 = 0; t0 < NTW; t0 += TG) {
                    float4 u[TG], v[TG];
#pragma unroll
                    for (int t = 0; t < TG; ++t) {
                        u[t] = *(const float4*)&T[(16 * bi[t0 + t] + c16) * TSS + 16 * sg + 4 * kq];
                        v[t] = *(const float4*)&T[(16 * bj[t0 + t] + c16) * TSS + 16 * sg + 4 * kq];
                    }
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].x, v[t].x, acc[t0 + t], 0, 0, 0);
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].y, v[t].y, acc[t0 + t], 0, 0, 0);
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].z, v[t].z, acc[t0 + t], 0, 0, 0);
#pragma unroll
                    for (int t = 0; t < TG; ++t) acc[t0 + t] = __builtin_amdgcn_mfma_f32_16x16x4f32(u[t].w, v[t].w, acc[t0 + t], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int t = 0; t < NTW; ++t)
#pragma unroll
            for (int e = 0; e < 4; ++e) dacc[t][e] += (double)acc[t][e];
    }
    // lane (c16, kq), register e of block (bi, bj) holds row 16 bi + 4 kq + e, column 16 bj + c16
#pragma unroll
    for (int t = 0; t < NTW; ++t) {
        int q = g + 4 * t;
        if (q >= a.ntile) q = -1;
        if constexpr (N16 == 5) {
            if (shared_operands) q = deal5_block(g, t);
        }
        if (q >= 0) {
            double* dst = a.ws + ((size_t)blockIdx.x * a.ntile + q) * 256 + si * 4;
#pragma unroll
            for (int e = 0; e < 4; ++e) dst[e] = dacc[t][e];
        }
    }
}

// Adds the workgroups' partial sums and scatters them into G (both triangles), b, hh;
// also stores the sample count.  Sixteen threads share an entry: thread p adds the
// partial sums of workgroups p, p + 16, ... in that order and the first thread then
// adds the sixteen results in order, so the sum depends on the launch shape only.
constexpr int RED_PARTS = 16, RED_ITEMS = NT / RED_PARTS;
__global__ __launch_bounds__(NT) void k_gram_reduce(const double* __restrict__ ws, int grid, int ntile, int n16, int L,
                                                    double M, double* __restrict__ normal) {
    __shared__ double part_sum[RED_PARTS][RED_ITEMS];
    const int item = threadIdx.x % RED_ITEMS, part = threadIdx.x / RED_ITEMS;
    const int idx = blockIdx.x * RED_ITEMS + item;      // ntile * 256 entries, a multiple of RED_ITEMS
    if (idx == 0 && part == 0) normal[(size_t)L * L + L + 1] = M;
    const int q = idx >> 8, lane = (idx >> 2) & 63, e = idx & 3;
    int bi, bj;
    block_of(q, n16, bi, bj);
    const int row = 16 * bi + 4 * (lane >> 4) + e, col = 16 * bj + (lane & 15);
    const bool wanted = row <= col && col <= L;         // diagonal blocks hold both triangles: keep the upper one
    double sum = 0.0;
    if (wanted)
        for (int w = part; w < grid; w += RED_PARTS) sum += ws[((size_t)w * ntile + q) * 256 + (idx & 255)];
    part_sum[part][item] = sum;
    __syncthreads();
    if (part != 0 || !wanted) return;
    for (int p = 1; p < RED_PARTS; ++p) sum += part_sum[p][item];
    if (col < L) {
        normal[(size_t)row * L + col] = sum;
        normal[(size_t)col * L + row] = sum;
    } else {
        if (row < L) normal[(size_t)L * L + row] = sum;
        else normal[(size_t)L * L + L] = sum;   // row == col == L: h^T h
    }
}

size_t tensor_elems(const sr_tensor* t) { return (size_t)t->n * t->c * t->h * t->w; }

// ---------------------------------------------------------------------------
// Host side of Alg. 1 (section III-A).
//
// The atoms keep their numbers throughout: what a round removes is a flag, and the
// rescaling of the kept atoms' coefficients by the regression scales (Eq. 9; the
// stand-in for fine-tuning the network between rounds) is a per-atom factor that
// multiplies the normal equations where they are read, G'_ij = c_i c_j G_ij and
// b'_i = c_i b_i.  Nothing is copied or rewritten between rounds.
// ---------------------------------------------------------------------------
struct SelectionProblem {
    const double* G;            // L x L, row-major
    const double* b;            // L
    int L;
    double M;                   // samples behind the normal equations
    std::vector<double> scale;  // c_i
    std::vector<char> alive;    // atoms still in the dictionary

    double g(int i, int j) const { return scale[i] * scale[j] * G[(size_t)i * L + j]; }
    double rhs(int i) const { return scale[i] * b[i]; }
};

// Minimiser of (1/M) |h - R w|^2 + lambda |w|_1 over the living atoms (Eq. 7), from the normal
// equations.  Coordinate descent in the "covariance" form: the correlations of the residual with every
// atom, corr_i = b'_i - sum_j G'_ij w_j, are kept up to date, so that a coordinate costs O(1) to
// examine and O(L) only when it moves.  Passes alternate between all living atoms and the current
// support, as long as a pass over all of them still moves something.  `w` is the starting point (any;
// the problem is convex) and receives the result; coordinates at zero are exact zeros.
class LassoSolver {
public:
    explicit LassoSolver(const SelectionProblem& p) : p_(p), corr_(p.L) {}

    int solve(double lambda, std::vector<double>& w) {
        const double threshold = 0.5 * lambda * p_.M;
        members_.clear();
        for (int i = 0; i < p_.L; ++i) {
            if (p_.alive[i]) members_.push_back(i);
            else w[i] = 0.0;
        }
        for (int i : members_) {
            double c = p_.rhs(i);
            for (int j : members_) c -= p_.g(i, j) * w[j];
            corr_[i] = c;
        }
        for (int round = 0; round < 100000; ++round) {
            if (!pass(members_, threshold, w)) break;          // nothing moved anywhere: the optimum
            support_.clear();
            for (int i : members_)
                if (w[i] != 0.0) support_.push_back(i);
            for (int inner = 0; inner < 100000 && pass(support_, threshold, w); ++inner) {}
        }
        int nonzero = 0;
        for (int i : members_) nonzero += w[i] != 0.0;
        return nonzero;
    }

private:
    // one pass over `which`; true if some weight moved by more than the tolerance
    bool pass(const std::vector<int>& which, double threshold, std::vector<double>& w) {
        double moved = 0.0, largest = 1.0;
        for (int j : which) {
            const double gjj = p_.g(j, j);
            double target = 0.0;
            if (gjj > 0.0) {
                const double z = corr_[j] + gjj * w[j];            // correlation with atom j left out
                if (z > threshold) target = (z - threshold) / gjj;
                else if (z < -threshold) target = (z + threshold) / gjj;
            }
            const double step = target - w[j];
            if (step != 0.0) {
                for (int i : members_) corr_[i] -= p_.g(i, j) * step;
                w[j] = target;
                moved = fmax(moved, fabs(step));
            }
            largest = fmax(largest, fabs(target));
        }
        return moved > 1e-13 * largest;
    }

    const SelectionProblem& p_;
    std::vector<double> corr_;
    std::vector<int> members_, support_;
};

// Regression scales of the atoms in `set` (Eq. 9): the least-squares fit of the target by their
// responses, G'_SS x = b'_S.  Cholesky factorisation; a pivot that vanishes (responses that are
// linearly dependent on earlier ones) leaves that atom's scale at zero.
std::vector<double> regression_scales(const SelectionProblem& p, const std::vector<int>& set) {
    const int m = (int)set.size();
    std::vector<double> C((size_t)m * m, 0.0), x(m, 0.0);
    std::vector<char> dropped(m, 0);
    for (int i = 0; i < m; ++i) {
        for (int j = 0; j <= i; ++j) {
            double v = p.g(set[i], set[j]);
            for (int k = 0; k < j; ++k) v -= C[(size_t)i * m + k] * C[(size_t)j * m + k];
            if (i == j) {
                const double floor = 1e-13 * p.g(set[i], set[i]);
                if (v > floor && v > 0.0) C[(size_t)i * m + i] = sqrt(v);
                else dropped[i] = 1;
            } else {
                C[(size_t)i * m + j] = dropped[j] ? 0.0 : v / C[(size_t)j * m + j];
            }
        }
    }
    for (int i = 0; i < m; ++i) {                     // forward: C y = b'
        if (dropped[i]) continue;
        double v = p.rhs(set[i]);
        for (int k = 0; k < i; ++k) v -= C[(size_t)i * m + k] * x[k];
        x[i] = v / C[(size_t)i * m + i];
    }
    for (int i = m - 1; i >= 0; --i) {                // backward: C^T x = y
        if (dropped[i]) { x[i] = 0.0; continue; }
        double v = x[i];
        for (int k = i + 1; k < m; ++k) v -= C[(size_t)k * m + i] * x[k];
        x[i] = v / C[(size_t)i * m + i];
    }
    return x;
}

}  // namespace

extern "C" __attribute__((visibility("default")))
size_t sr_atom_gram_workspace_bytes(int L) {
    if (L < 1 || L > SR_SELECT_MAX_ATOMS) return 0;
    return (size_t)GRID * upper_blocks(column_blocks(L)) * 256 * sizeof(double);
}

namespace {

// Scratch of the entry point that allocates nothing: the per-workgroup partial sums of up to
// SR_SELECT_STATIC_MAX_ATOMS atoms (five column blocks: 512 workgroups x 15 blocks x 256 doubles,
// 15 MiB).  Every GPU the library runs on holds its own copy until the process ends.  In host
// code the array's name is only a stand-in for the symbol: its device address is asked for once
// per device, with that device current, and everything below uses that address.
constexpr size_t STATIC_SCRATCH_DOUBLES = (size_t)512 * 15 * 256;
static __device__ __align__(256) double static_scratch[STATIC_SCRATCH_DOUBLES];

std::mutex static_scratch_lock;
double* static_scratch_addr[64];          // by device ordinal

hipError_t static_scratch_of_current_device(double** out) {
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64) return hipErrorInvalidDevice;
    std::lock_guard<std::mutex> hold(static_scratch_lock);
    if (!static_scratch_addr[dev]) {
        void* p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(static_scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        static_scratch_addr[dev] = (double*)p;
    }
    *out = static_scratch_addr[dev];
    return hipSuccess;
}

int atom_gram(const sr_tensor* up, const sr_tensor* coeff, const sr_tensor* dict, const sr_tensor* target,
              int L, int k, int channels, int stride, void* workspace, size_t workspace_bytes,
              double* normal, void* stream);

}  // namespace

extern "C" __attribute__((visibility("default")))
int sr_atom_gram(const sr_tensor* up, const sr_tensor* coeff, const sr_tensor* dict, const sr_tensor* target,
                 int L, int k, int channels, int stride, void* workspace, size_t workspace_bytes,
                 double* normal, void* stream) {
    return atom_gram(up, coeff, dict, target, L, k, channels, stride, workspace, workspace_bytes, normal, stream);
}

extern "C" __attribute__((visibility("default")))
int sr_atom_gram_static(const sr_tensor* up, const sr_tensor* coeff, const sr_tensor* dict, const sr_tensor* target,
                        int L, int k, int channels, int stride, double* normal, void* stream) {
    if (L < 1 || L > SR_SELECT_MAX_ATOMS) return SR_ERR_UNSUPPORTED;
    if (L > SR_SELECT_STATIC_MAX_ATOMS || sr_atom_gram_workspace_bytes(L) > STATIC_SCRATCH_DOUBLES * sizeof(double))
        return SR_ERR_SCRATCH;
    double* scratch = nullptr;
    if (static_scratch_of_current_device(&scratch) != hipSuccess) return SR_ERR_LAUNCH;
    return atom_gram(up, coeff, dict, target, L, k, channels, stride, scratch, STATIC_SCRATCH_DOUBLES * sizeof(double),
                     normal, stream);
}

namespace {

int atom_gram(const sr_tensor* up, const sr_tensor* coeff, const sr_tensor* dict, const sr_tensor* target,
              int L, int k, int channels, int stride, void* workspace, size_t workspace_bytes,
              double* normal, void* stream) {
    if (!up || !coeff || !dict || !target || !normal) return SR_ERR_NULL;
    if (up->dtype != SR_F32 || target->dtype != SR_F32 || dict->dtype != SR_F32 ||
        (coeff->dtype != SR_F32 && coeff->dtype != SR_F16 && coeff->dtype != SR_F8E4M3 && coeff->dtype != SR_BF16))
        return SR_ERR_UNSUPPORTED;
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
            (uintptr_t)coeff->data % (coeff->dtype == SR_F32 ? 4 : (coeff->dtype == SR_F8E4M3 ? 1 : 2))) return SR_ERR_ALIGN;
    }
    GramArgs a;
    a.up = (const float*)up->data; a.coeff = coeff->data; a.dict = (const float*)dict->data;
    a.target = (const float*)target->data; a.ws = (double*)workspace;
    a.N = up->n; a.C = channels; a.H = up->h; a.W = up->w; a.L = L; a.stride = stride;
    a.ny = empty ? 0 : (up->h + stride - 1) / stride;
    a.nx = empty ? 0 : (up->w + stride - 1) / stride;
    a.n16 = column_blocks(L);
    a.ntile = upper_blocks(a.n16);
    const hipStream_t st = (hipStream_t)stream;
    // staged row segments (32-bit offsets within a plane; LDS for the tiles), else per-lane gathers
    const bool rows_ok = stride <= STMAX && (int64_t)up->h * up->w < (1 << 30);
    bool rows = false;
    int grid = GRID;
#define SR_GRAM_LAUNCH_N(KS, TC, N16)                                                                      \
    do {                                                                                                    \
        const size_t lds = rows_lds_floats(KS, N16, channels) * sizeof(float);                              \
        rows = rows_ok && lds <= 160 * 1024;                                                                \
        if (rows) {                                                                                         \
            if (lds > 65536 &&                                                                              \
                hipFuncSetAttribute((const void*)k_atom_gram_rows<KS, TC, N16>,                             \
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds) != hipSuccess)    \
                return SR_ERR_LAUNCH;                                                                       \
            grid = ((N16) <= 5 && (KS) <= 5 && 2 * lds <= 160 * 1024) ? 2 * GRID2 : GRID2;                  \
            hipLaunchKernelGGL((k_atom_gram_rows<KS, TC, N16>), dim3(grid), dim3(NT2), lds, st, a);         \
        } else {                                                                                            \
            hipLaunchKernelGGL((k_atom_gram<KS, TC, N16>), dim3(GRID), dim3(NT), 0, st, a);                 \
        }                                                                                                   \
    } while (0)
#define SR_GRAM_LAUNCH_T(KS, TC)                                                                           \
    do {                                                                                                    \
        if (a.n16 <= 2) SR_GRAM_LAUNCH_N(KS, TC, 2);                                                        \
        else if (a.n16 <= 5) SR_GRAM_LAUNCH_N(KS, TC, 5);                                                   \
        else SR_GRAM_LAUNCH_N(KS, TC, 9);                                                                   \
    } while (0)
#define SR_GRAM_LAUNCH(KS)                                                                                  \
    do {                                                                                                    \
        if (coeff->dtype == SR_F16) SR_GRAM_LAUNCH_T(KS, __half);                                           \
        else if (coeff->dtype == SR_F32) SR_GRAM_LAUNCH_T(KS, float);                                       \
        else if (coeff->dtype == SR_BF16) SR_GRAM_LAUNCH_T(KS, bf16v);                                      \
        else SR_GRAM_LAUNCH_T(KS, e4m3);                                                                    \
    } while (0)
    switch (k) {
    case 3:  SR_GRAM_LAUNCH(3); break;
    case 5:  SR_GRAM_LAUNCH(5); break;
    default: SR_GRAM_LAUNCH(7); break;
    }
#undef SR_GRAM_LAUNCH
#undef SR_GRAM_LAUNCH_T
#undef SR_GRAM_LAUNCH_N
    if (hipGetLastError() != hipSuccess) return SR_ERR_LAUNCH;
    const double M = (double)a.N * a.ny * a.nx * a.C;
    const int items = a.ntile * 256;
    hipLaunchKernelGGL(k_gram_reduce, dim3(items / RED_ITEMS), dim3(NT), 0, st,
                       (const double*)workspace, grid, a.ntile, a.n16, L, M, normal);
    return hipGetLastError() == hipSuccess ? SR_OK : SR_ERR_LAUNCH;
}

}  // namespace

extern "C" __attribute__((visibility("default")))
int sr_select_atoms(const double* normal, int L, double alpha, double delta_alpha, double lambda0, double eps,
                    int* kept, int* n_kept, float* gamma, double* lambda_out) {
    if (!normal || !kept || !n_kept || !gamma) return SR_ERR_NULL;
    if (L < 1 || L > SR_SELECT_MAX_ATOMS || !(alpha > 0.0) || alpha > 1.0 || !(delta_alpha > 0.0) ||
        !(lambda0 > 0.0) || !(eps >= 0.0)) return SR_ERR_UNSUPPORTED;
    SelectionProblem prob;
    prob.G = normal;
    prob.b = normal + (size_t)L * L;
    prob.L = L;
    prob.M = normal[(size_t)L * L + L + 1];
    if (!(prob.M > 0.0)) return SR_ERR_UNSUPPORTED;
    prob.scale.assign(L, 1.0);
    prob.alive.assign(L, 1);
    LassoSolver lasso(prob);
    int living = L;
    double lam = lambda0, fraction = 1.0;
    std::vector<double> w(L), trial(L);
    // Alg. 1: the kept fraction comes down in steps of delta_alpha; each step finds, by doubling and then
    // bisection, a lambda whose LASSO solution keeps no more atoms than the step allows, removes the atoms
    // at zero, and refits the scales of the others.
    while (fraction > alpha + 1e-12 && living > 0) {
        fraction = fmax(alpha, fraction - delta_alpha);
        const double allowed = fraction * L;
        // every solve starts from all weights at one: the dictionary as it stands, nothing selected yet
        auto support_at = [&](double lambda, std::vector<double>& weights) {
            std::fill(weights.begin(), weights.end(), 1.0);
            return lasso.solve(lambda, weights);
        };
        double too_many = 0.5 * lam, few_enough = lam;         // the bracket on lambda
        int count = support_at(few_enough, w);
        while (count > allowed) {
            too_many = few_enough;
            few_enough *= 2.0;
            count = support_at(few_enough, w);
        }
        // the count may have dropped further than asked: look between the two for a lambda that keeps more,
        // but still few enough
        for (int halvings = 0; halvings < 60; ++halvings) {
            if (allowed - count < 1.0 || fabs(allowed - count) <= eps * L) break;
            const double middle = 0.5 * (too_many + few_enough);
            const int c = support_at(middle, trial);
            if (c > allowed) {
                too_many = middle;
            } else {
                few_enough = middle;
                count = c;
                w.swap(trial);
            }
        }
        lam = few_enough;
        std::vector<int> survivors;
        for (int i = 0; i < L; ++i) {
            if (prob.alive[i] && w[i] != 0.0) survivors.push_back(i);
            else prob.alive[i] = 0;
        }
        living = (int)survivors.size();
        if (living == 0) break;
        const std::vector<double> fit = regression_scales(prob, survivors);
        for (int i = 0; i < living; ++i) prob.scale[survivors[i]] *= fit[i];
    }
    int n = 0;
    for (int i = 0; i < L; ++i)
        if (prob.alive[i] && living > 0) { kept[n] = i; gamma[n] = (float)prob.scale[i]; ++n; }
    *n_kept = n;
    if (lambda_out) *lambda_out = lam;
    return SR_OK;
}
